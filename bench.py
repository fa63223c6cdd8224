#!/usr/bin/env python3
"""Benchmark of the KV Packet serving hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic requests: one
kvp_assemble launch covering every layer, then kvp_query_prefill for each layer.  Inputs
(packet store, Q / K_new / V_new of every layer) are resident in HBM before the timed
region.  Prints ONE JSON line: the metric's 8K-context point as the headline (value,
roofline of the whole step, of the per-layer attention launches and of the gather, the CPU
oracle's time, parity of a sampled layer), then -- in the default run -- a `configs` list with
a short measurement and a parity check of every other workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PCIE_PEAK_GBS = 63.0     # PCIe 5.0 x16, one direction
HBM_PEAK_GBS = 8000.0
BF16_PEAK_TFLOPS = 2500.0
F32_VALU_PEAK_TFLOPS = 157.3
TOL = {"f32": 1e-5, "bf16": 2e-2}   # attention: max abs error against the oracle

T_START = time.perf_counter()


def note(what):  # progress on stderr: a profiled run is slow, not silent
    print("[%7.2f s] %s" % (time.perf_counter() - T_START, what), file=sys.stderr, flush=True)


def measured_traffic(name):
    """HBM bytes from the committed rocprofv3 --pmc summary profiles/<name>_pmc.txt (FETCH_SIZE +
    WRITE_SIZE, scaled by a plain copy of known size): its `traffic_bytes_per_launch:` line, or None."""
    path = os.path.join(ROOT, "profiles", "%s_pmc.txt" % name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


WORKLOADS = {
    "llama_8k": lambda W: W.llama_8k(),
    "llama_8k_decode": lambda W: W.llama_8k_decode(),
    "llama_8k_pruned": lambda W: W.llama_8k_pruned(),                     # packets pruned offline, per layer (Sec. 5.4)
    "llama_k5": lambda W: W.llama_k5(),
    "qwen_k20": lambda W: W.qwen_k20(),
    "llama_long_b8": lambda W: W.llama_long_b8(n_layers=4),
    "llama_long_b8_q32": lambda W: W.llama_long_b8(n_layers=4, n_q=32),   # the same contexts, HBM-bound (n_q g = 128)
    "llama_long_b8_q1": lambda W: W.llama_long_b8(n_layers=4, n_q=1),     # one decode step over them
    "serving_mix": lambda W: W.serving_mix(n_layers=1),
    "tiny_fp32": lambda W: W.tiny_fp32(),
}


def make_workload(name):
    import kvp_workloads as W
    w = WORKLOADS[name](W)
    w.name = name
    return w


# ------------------------------------------------------------------------------------
# CPU oracle: timing (cpu_baseline) and parity of a sampled request / layer.  The only
# part of this file that touches oracle/.
# ------------------------------------------------------------------------------------
def cpu_baseline(w, sample_layers):
    """Times the CPU oracle, as it stands, on `sample_layers` layers of request 0."""
    import numpy as np
    import kvp_workloads as W
    import oracle
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    rq = w.requests[0]
    if w.prune is not None:
        return cpu_baseline_pruned(w, sample_layers, f)
    pk, pv = [], []
    for p in rq.packet_ids:
        k, v = w.packet_kv(p, layers=sample_layers)
        pk.append(W.to_numpy(k)), pv.append(W.to_numpy(v))
    rows = w.ctx_len(0) + rq.n_q
    npdt = np.float32 if w.dtype == "f32" else np.uint16
    ko = np.zeros((sample_layers, w.n_kv_heads, rows, w.head_dim), npdt)
    vo = np.zeros_like(ko)
    qs = [tuple(W.to_numpy(x) for x in w.query(0, l)) for l in range(sample_layers)]
    t0 = time.perf_counter()
    ko, vo, ctx = oracle.assemble(w.dtype, pk, pv, f, rq.base_pos, rows, ko, vo)
    t1 = time.perf_counter()
    for l in range(sample_layers):
        q, kn, vn = qs[l]
        oracle.query_prefill(w.dtype, q, kn, vn, f, ctx, ko[l], vo[l])
    t2 = time.perf_counter()
    return dict(value=(t2 - t0) * 1e6 / sample_layers, unit="us/layer", cores=oracle.num_threads(),
                kind="oracle",
                sample="request 0, %d of %d layers of %s (assemble %.0f us/layer, prefill %.0f us/layer)"
                % (sample_layers, w.n_layers, w.name, (t1 - t0) * 1e6 / sample_layers,
                   (t2 - t1) * 1e6 / sample_layers))


def cpu_baseline_pruned(w, sample_layers, f):
    """The same for a pruned workload: the oracle composes and attends layer by layer."""
    import numpy as np
    import kvp_workloads as W
    import oracle
    rq = w.requests[0]
    spans = [int(w.packet_lens[p]) for p in rq.packet_ids]
    kv = [tuple(W.to_numpy(x) for x in w.packet_kv(p, layers=sample_layers)) for p in rq.packet_ids]
    ins = []
    for l in range(sample_layers):
        keep = [w.kept_rows(p, l) for p in rq.packet_ids]
        ins.append(([np.ascontiguousarray(k[l][:, s_]) for (k, _), s_ in zip(kv, keep)],
                    [np.ascontiguousarray(v[l][:, s_]) for (_, v), s_ in zip(kv, keep)],
                    tuple(W.to_numpy(x) for x in w.query(0, l))))
    t_asm = t_pre = 0.0
    for ks, vs, (q, kn, vn) in ins:
        t0 = time.perf_counter()
        ko, vo, rows, pos_end = oracle.assemble_layer_spans(w.dtype, ks, vs, spans, f, rq.base_pos,
                                                            t_cap=sum(k.shape[1] for k in ks) + rq.n_q)
        t1 = time.perf_counter()
        oracle.query_prefill_at(w.dtype, q, kn, vn, f, rows, pos_end, ko, vo)
        t2 = time.perf_counter()
        t_asm += t1 - t0
        t_pre += t2 - t1
    return dict(value=(t_asm + t_pre) * 1e6 / sample_layers, unit="us/layer", cores=oracle.num_threads(),
                kind="oracle",
                sample="request 0, %d of %d layers of %s (assemble %.0f us/layer, prefill %.0f us/layer)"
                % (sample_layers, w.n_layers, w.name, t_asm * 1e6 / sample_layers, t_pre * 1e6 / sample_layers))


def parity(run, request=0, layer=0):
    """The state the timed steps left on the GPU, against the oracle, for one request and layer:
    are the cache rows (assembled rows and appended query rows) the oracle's bits, and how far is
    the attention output from the oracle's (maximum absolute error over the request's rows).  The
    in-place path has no cache: there the rotated K_new rows it hands back are compared."""
    import numpy as np
    import torch
    import kvp_workloads as W
    import oracle
    w, r = run["w"], request
    rq = w.requests[r]
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    q, kn, vn = (W.to_numpy(x) for x in w.query(r, layer))
    lo, hi = int(run["q_off"][r]), int(run["q_off"][r + 1])
    # one more call on that layer, so that `out` holds its result (the steps end on the last layer)
    out = torch.full_like(run["qkv"][layer][0], float("nan"))
    run["call_layer"](layer, out)
    torch.cuda.synchronize()
    got = out[lo:hi].float().cpu().numpy().astype(np.float64)
    if w.prune is None:
        pk, pv = [], []
        for p in rq.packet_ids:
            k, v = w.packet_kv(p, layers=layer + 1)     # (the draws of a layer do not depend on the depth asked for)
            pk.append(np.ascontiguousarray(W.to_numpy(k)[layer:layer + 1]))
            pv.append(np.ascontiguousarray(W.to_numpy(v)[layer:layer + 1]))
        rows = w.ctx_len(r) + rq.n_q
        npdt = np.float32 if w.dtype == "f32" else np.uint16
        ko = np.zeros((1, w.n_kv_heads, rows, w.head_dim), npdt)
        vo = np.zeros_like(ko)
        ko, vo, ctx = oracle.assemble(w.dtype, pk, pv, f, rq.base_pos, rows, ko, vo)
        ref = oracle.query_prefill(w.dtype, q, kn, vn, f, ctx, ko[0], vo[0])
        ko, vo = ko[0], vo[0]
    else:
        spans = [int(w.packet_lens[p]) for p in rq.packet_ids]
        ks, vs = [], []
        for p in rq.packet_ids:
            k, v = w.packet_kv(p, layers=layer + 1)
            keep = w.kept_rows(p, layer)
            ks.append(np.ascontiguousarray(W.to_numpy(k)[layer][:, keep]))
            vs.append(np.ascontiguousarray(W.to_numpy(v)[layer][:, keep]))
        ko, vo, ctx, pos_end = oracle.assemble_layer_spans(w.dtype, ks, vs, spans, f, rq.base_pos,
                                                           t_cap=sum(k.shape[1] for k in ks) + rq.n_q)
        ref = oracle.query_prefill_at(w.dtype, q, kn, vn, f, ctx, pos_end, ko, vo)
        rows = ctx + rq.n_q
    if run["path"] == "cache":
        k_gpu, v_gpu = run["cache"].logical(r, layer, rows)
        exact = bool(np.array_equal(W.to_numpy(k_gpu), ko[:, :rows]) and np.array_equal(W.to_numpy(v_gpu), vo[:, :rows]))
        what = "cache rows 0..%d (assembled + appended)" % (rows - 1)
    else:
        tail = W.to_numpy(run["k_tail"][lo:hi])                                 # [n_q][Hkv][d]
        exact = bool(np.array_equal(tail.transpose(1, 0, 2), ko[:, ctx:ctx + rq.n_q]))
        what = "rotated K_new rows (no cache is built)"
    err = float(np.max(np.abs(got - ref))) if rq.n_q else 0.0
    return {"request": r, "layer": layer, "bit_exact": exact, "bit_exact_what": what,
            "attention_max_abs_err": err, "tolerance": TOL[w.dtype], "ok": bool(exact and err <= TOL[w.dtype])}


# ------------------------------------------------------------------------------------
def setup(w, args, all_packets=False):
    """Store, cache, workspace and inputs of workload `w` on the GPU, and its step function."""
    import numpy as np
    import torch
    import paper_2604_13226_amd as kvp
    from kvp_setup import build_store, make_cache

    dev = "cuda:0"
    if args.layers > 0:
        w.n_layers = min(w.n_layers, args.layers)
    if args.layout:
        w.paged = args.layout == "paged"
    w.shared_header = bool(args.shared_header)
    n_req = len(w.requests)
    whole = all_packets and len(w.packet_lens) <= 256 and args.store == "device"
    store = build_store(w, kvp, dev, packets=list(range(len(w.packet_lens))) if whole else None, arena=args.store,
                        progress=lambda i, n: print("store: packet %d of %d" % (i, n), file=sys.stderr, flush=True))
    cache = make_cache(w, kvp, store, dev, block_order=args.block_order, t_slack=0)
    reqs = [(rq.packet_ids, rq.base_pos) for rq in w.requests]
    q_off = np.zeros(n_req + 1, np.int32)
    for r in range(n_req):
        q_off[r + 1] = q_off[r] + w.requests[r].n_q
    tot_q = int(q_off[-1])
    ctx = [w.ctx_len(r) for r in range(n_req)]
    max_ctx = max(c + rq.n_q for c, rq in zip(ctx, w.requests))
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, n_req, tot_q, max_ctx), dev)
    qkv = []
    for layer in range(w.n_layers):
        parts = [w.query(r, layer, dev) for r in range(n_req)]
        qkv.append(tuple(torch.cat([p[i] for p in parts]).contiguous() for i in range(3)))
    out = torch.empty_like(qkv[0][0])
    k_tail = torch.empty_like(qkv[0][1])
    reqs0 = [(rq.packet_ids, 0) for rq in w.requests]
    torch.cuda.synchronize()

    pipelined = args.pipeline and args.path == "cache"
    if pipelined:
        # layer l is assembled on a side stream (default priority) while layer l-1 is attended
        # to; ready[l] orders prefill(l) behind assemble(l), free[l] orders the next step's
        # assemble(l) behind this step's prefill(l)
        side = torch.cuda.Stream()
        main = torch.cuda.current_stream()
        ready = [torch.cuda.Event() for _ in range(w.n_layers)]
        free = [torch.cuda.Event() for _ in range(w.n_layers)]
        for e in free:
            e.record(main)

    def call_layer(layer, dst):
        q, kn, vn = qkv[layer]
        if args.path == "cache":
            kvp.kvp_query_prefill(store, cache, layer, q, kn, vn, q_off, ws, dst)
        else:
            kvp.kvp_prefill_packets(store, reqs0, layer, q, kn, vn, q_off, k_tail, ws, dst)

    def step(ev=None):
        if ev:
            ev[0].record()
        if pipelined:
            G = max(1, args.pipeline_group)
            for l0 in range(0, w.n_layers, G):       # every group's assembly is queued on the side stream at once
                l1 = min(w.n_layers, l0 + G)
                side.wait_event(free[l1 - 1])
                kvp.kvp_assemble(store, reqs, cache, l0, l1, stream=side)
                ready[l0].record(side)
            for layer in range(w.n_layers):
                if layer % G == 0:
                    main.wait_event(ready[layer])
                call_layer(layer, out)
                if layer % G == G - 1 or layer == w.n_layers - 1:   # (only a group's last layer is waited for)
                    free[layer].record(main)
            if ev:
                ev[1].record()
                ev[2].record()
            return
        if args.path == "cache":
            kvp.kvp_assemble(store, reqs, cache)
        if ev:
            ev[1].record()
        for layer in range(w.n_layers):
            call_layer(layer, out)
        if ev:
            ev[2].record()

    return dict(kvp=kvp, w=w, dev=dev, store=store, cache=cache, reqs=reqs, q_off=q_off, tot_q=tot_q, ctx=ctx,
                ws=ws, qkv=qkv, out=out, k_tail=k_tail, step=step, call_layer=call_layer, pipelined=pipelined,
                path=args.path, n_req=n_req)


def time_steps(run, steps, warmup):
    """`warmup` untimed steps, then `steps` timed ones: wall clock between two device
    synchronisations, and HIP events (on the launch stream) around the assembly and around the
    layers' prefill calls of every timed step."""
    import numpy as np
    import torch
    step = run["step"]
    for i in range(warmup):
        step()
        if i == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return dict(ms_per_step=(t1 - t0) * 1e3 / steps,
                asm_ms=float(np.mean([e[0].elapsed_time(e[1]) for e in events])),
                pre_ms=float(np.mean([e[1].elapsed_time(e[2]) for e in events])),
                step_ms=np.array([e[0].elapsed_time(e[2]) for e in events]))


def figures(run, t):
    """Algorithmic bytes / flops of the workload and what the measured times make of them."""
    w, n_req = run["w"], run["n_req"]
    tok_bytes = w.kv_bytes_per_token_layer()
    # rows[l][r]: context rows of request r in layer l (the same in every layer unless pruned)
    rows = [[w.layer_rows(r, l) for r in range(n_req)] for l in range(w.n_layers if w.prune else 1)]
    if not w.prune:
        rows = rows * w.n_layers
    asm_bytes = 2.0 * tok_bytes * sum(c - rq.base_pos for rl in rows for c, rq in zip(rl, w.requests))  # read + write every K/V row
    pre_bytes = sum((c + rq.n_q) * tok_bytes for rl in rows for c, rq in zip(rl, w.requests)) / w.n_layers   # per layer
    pre_flops = sum(4.0 * rq.n_q * c * w.n_q_heads * w.head_dim
                    + 2.0 * rq.n_q * rq.n_q * w.n_q_heads * w.head_dim
                    for rl in rows for c, rq in zip(rl, w.requests)) / w.n_layers                           # per layer
    ms_per_step, asm_ms, pre_ms = t["ms_per_step"], t["asm_ms"], t["pre_ms"]
    if run["pipelined"]:  # the two overlap: only the whole step is observable
        asm_ms, pre_ms = ms_per_step, ms_per_step
    if run["path"] != "cache":
        asm_bytes = 0.0
    pre_us = pre_ms * 1e3 / w.n_layers
    f = dict(asm_bytes=asm_bytes, pre_bytes=pre_bytes, pre_flops=pre_flops, asm_us=asm_ms * 1e3, pre_us=pre_us,
             asm_gbs=asm_bytes / (max(asm_ms, 1e-6) * 1e-3) / 1e9,
             pre_gbs=pre_bytes / (pre_us * 1e-6) / 1e9, pre_tflops=pre_flops / (pre_us * 1e-6) / 1e12,
             step_bytes=asm_bytes + pre_bytes * w.n_layers, step_flops=pre_flops * w.n_layers)
    # HBM-bound while the packed query rows per KV head stay below the chip's flop-per-byte
    # balance, else bound by the bf16 matrix cores (the fp32 path: by the fp32 vector units)
    intensity = pre_flops / max(pre_bytes, 1.0)
    if w.dtype == "bf16" and intensity > BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS:
        f["pre_roofline"] = {"bound": "mfma", "achieved": f["pre_tflops"], "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": f["pre_tflops"] / BF16_PEAK_TFLOPS}
    elif w.dtype == "f32" and intensity > F32_VALU_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS:
        f["pre_roofline"] = {"bound": "alu", "achieved": f["pre_tflops"], "peak": F32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": f["pre_tflops"] / F32_VALU_PEAK_TFLOPS}
    else:
        f["pre_roofline"] = {"bound": "hbm", "achieved": f["pre_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": f["pre_gbs"] / HBM_PEAK_GBS}
    # the whole step: the time its algorithmic bytes take at HBM peak plus, for compute-bound
    # prefill, the time its flops take at the matrix peak beyond that -- over the measured time
    floor_us = f["asm_bytes"] / (HBM_PEAK_GBS * 1e3) + w.n_layers * max(
        pre_bytes / (HBM_PEAK_GBS * 1e3),
        pre_flops / (BF16_PEAK_TFLOPS * 1e6) if w.dtype == "bf16" else pre_flops / (F32_VALU_PEAK_TFLOPS * 1e6))
    f["floor_us_per_layer"] = floor_us / w.n_layers
    f["step_frac_of_floor"] = floor_us / (ms_per_step * 1e3)
    return f


def config_record(name, args, steps, warmup, path="cache", per_request=False):
    """A short measurement + parity check of one more workload, for the `configs` list."""
    import torch
    a = argparse.Namespace(**vars(args))
    a.path, a.store, a.pipeline, a.layers, a.layout, a.shared_header = path, "device", False, 0, "", False
    w = make_workload(name)
    run = setup(w, a)
    t = time_steps(run, steps, warmup)
    f = figures(run, t)
    rec = {"workload": name, "path": path, "layers": w.n_layers, "requests": run["n_req"],
           "ctx": run["ctx"][:2], "n_q": [rq.n_q for rq in w.requests[:2]],
           "layout": "paged" if w.paged else "contiguous", "dtype": w.dtype,
           "us_per_layer": t["ms_per_step"] * 1e3 / w.n_layers,
           "assemble": {"us_per_launch": f["asm_us"], "bytes": f["asm_bytes"], "GBs": f["asm_gbs"],
                        "hbm_frac": f["asm_gbs"] / HBM_PEAK_GBS} if path == "cache" else None,
           "prefill": dict(f["pre_roofline"], us_per_layer=f["pre_us"], bytes_per_layer=f["pre_bytes"],
                           flops_per_layer=f["pre_flops"]),
           "floor_us_per_layer": f["floor_us_per_layer"], "frac_of_floor": f["step_frac_of_floor"],
           "steps": steps, "warmup": warmup}
    if run["n_req"] > 1:
        rec["tokens_per_s"] = (sum(run["ctx"]) + run["tot_q"]) / (t["ms_per_step"] * 1e-3)
    if per_request:
        rec["per_request"] = per_request_latency(run, args, mixes=1)
    r = 0
    if run["n_req"] > 1:   # a request of middling size: the oracle's naive attention stays within seconds
        order = sorted(range(run["n_req"]), key=lambda i: run["ctx"][i] * max(w.requests[i].n_q, 1))
        r = order[len(order) // 2] if name == "serving_mix" else order[0]
    rec["parity"] = parity(run, request=r, layer=0)
    run["kvp"].kvp_store_destroy(run["store"])
    del run
    torch.cuda.empty_cache()
    note("config %s (%s) done" % (name, path))
    return rec


def per_request_latency(run, args, mixes=1):
    """Every request issued alone, back to back (closed loop): wall-clock latency of its
    kvp_assemble + kvp_query_prefill over the workload's layers.  A first, untimed pass loads
    every kernel variant; the timed pass then meets each request with no plan kept for it (the
    store keeps a handful of plans, the batch has many more geometries)."""
    import numpy as np
    import torch
    from kvp_setup import build_store, make_cache
    kvp, w, dev, ws = run["kvp"], run["w"], run["dev"], run["ws"]

    def latencies(wl, st, inputs, offsets):
        lat = []
        for timed in (False, True):
            for r, rq in enumerate(wl.requests):
                if rq.n_q == 0:
                    continue
                wr = type(wl)(**{**wl.__dict__, "requests": [rq]})
                c1 = make_cache(wr, kvp, st, dev, t_slack=0)
                qo1 = np.array([0, rq.n_q], np.int32)
                parts = [tuple(x[offsets[r]:offsets[r + 1]].contiguous() for x in inputs[layer]) for layer in range(wl.n_layers)]
                o1 = torch.empty_like(parts[0][0])
                torch.cuda.synchronize()
                t_a = time.perf_counter()
                kvp.kvp_assemble(st, [(rq.packet_ids, rq.base_pos)], c1)
                for layer in range(wl.n_layers):
                    q1, k1, v1 = parts[layer]
                    kvp.kvp_query_prefill(st, c1, layer, q1, k1, v1, qo1, ws, o1)
                torch.cuda.synchronize()
                if timed:
                    lat.append((time.perf_counter() - t_a) * 1e6)
        return lat
    lat = latencies(w, run["store"], run["qkv"], run["q_off"])
    n_mixes = 1
    for mix in range(1, max(1, mixes)):   # the same recipe under other seeds
        import kvp_workloads as W
        if w.name != "serving_mix":
            break
        wm = W.serving_mix(seed=w.seed + mix, n_layers=w.n_layers)
        wm.paged, wm.shared_header = w.paged, w.shared_header
        sm = build_store(wm, kvp, dev)
        om = np.concatenate([[0], np.cumsum([rq.n_q for rq in wm.requests])]).astype(np.int32)
        inputs = []
        for layer in range(wm.n_layers):
            parts = [wm.query(r, layer, dev) for r in range(len(wm.requests))]
            inputs.append(tuple(torch.cat([p_[i] for p_ in parts]).contiguous() for i in range(3)))
        lat += latencies(wm, sm, inputs, om)
        kvp.kvp_store_destroy(sm)
        del sm, inputs
        n_mixes += 1
        note("mix %d of %d timed" % (n_mixes, mixes))
    lat = np.array(lat)
    return {"n": int(len(lat)), "mixes": n_mixes, "p50_us": float(np.percentile(lat, 50)),
            "p99_us": float(np.percentile(lat, 99)), "mean_us": float(lat.mean()),
            "what": "one request at a time, each met without a kept plan: assemble + prefill over "
                    "%d layer(s), wall clock from the call to the end of the GPU work" % w.n_layers}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps first: the GPU clock takes some 20 ms of load to settle")
    ap.add_argument("--workload", default="llama_8k", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=0,
                    help="instantiate only this many layers of the workload (counter runs, where every "
                         "dispatch is slow, keep the store small with it)")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="timed steps only: no CPU oracle (timing, parity), no graph replay, no other "
                         "configs (the profiling commands use it)")
    ap.add_argument("--cpu-layers", type=int, default=16)
    ap.add_argument("--configs", default="auto", choices=["auto", "all", "none"],
                    help="after the headline, measure and check the other workloads too (auto: when the "
                         "headline is the default one, on the default path)")
    ap.add_argument("--config-steps", type=int, default=100)
    ap.add_argument("--config-warmup", type=int, default=50)
    ap.add_argument("--path", default="cache", choices=["cache", "packets"],
                    help="cache: kvp_assemble + kvp_query_prefill (the metric's path); packets: "
                         "kvp_prefill_packets, attention read in place from the store, no assembly")
    ap.add_argument("--store", default="device", choices=["device", "host"],
                    help="device: packet store in HBM (the metric's configuration); host: in pinned host "
                         "memory, read over PCIe at every assembly (the paper's tier; reported apart)")
    ap.add_argument("--pipeline", action="store_true",
                    help="assemble layer by layer on a second stream, under the previous layer's prefill")
    ap.add_argument("--pipeline-group", type=int, default=1,
                    help="with --pipeline: layers per assembly launch")
    ap.add_argument("--layout", default="", choices=["", "contiguous", "paged"],
                    help="cache layout (default: the workload's own); paged uses 16-row blocks in a seeded random order")
    ap.add_argument("--block-order", default="random", choices=["random", "sequential"],
                    help="paged layout: how the pool's blocks are dealt to the requests")
    ap.add_argument("--shared-header", action="store_true",
                    help="store the header rows once (kvp_store_put_header) and every packet without them")
    ap.add_argument("--mixes", type=int, default=1,
                    help="with --per-request on serving_mix: time the requests of this many reseeded mixes")
    ap.add_argument("--per-request", action="store_true",
                    help="batched workloads: also time every request alone (p50 / p99 latency)")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the extra measurement of the step replayed from a HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (a known-size kernel to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = make_workload(args.workload)
    run = setup(w, args, all_packets=True)
    kvp, store, n_req, ctx, tot_q = run["kvp"], run["store"], run["n_req"], run["ctx"], run["tot_q"]
    note("store, cache and inputs ready")
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=run["dev"])
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    t = time_steps(run, args.steps, args.warmup)
    note("timed steps done")
    f = figures(run, t)
    ms_per_step, step_ms = t["ms_per_step"], t["step_ms"]
    pipelined = run["pipelined"]

    n_attn = "%d x (attention + combine)" % w.n_layers
    roofline_assemble = {"bound": "hbm", "kernel": "assemble_vec_kernel (all layers, one launch)",
                         "achieved": f["asm_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": f["asm_gbs"] / HBM_PEAK_GBS, "traffic": measured_traffic("assemble_" + w.name),
                         "bytes_per_launch": f["asm_bytes"], "us_per_launch": f["asm_us"]}
    # the launches that take most of the step's time: each layer's attention kernel and the
    # combine kernel behind it, timed together (HIP events around all layers' calls)
    roofline_attention = dict(f["pre_roofline"], kernel="attention_mfma_kernel + combine kernel, per layer",
                              traffic=measured_traffic("attention_" + w.name),
                              bytes_per_launch=f["pre_bytes"], flops_per_launch=f["pre_flops"], us_per_launch=f["pre_us"])
    # the metric's path as a whole: every algorithmic byte of the step over the step's time
    step_gbs = f["step_bytes"] / (ms_per_step * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": ("whole step: assemble_vec_kernel + " + n_attn) if args.path == "cache" else
                ("whole step: " + n_attn + ", packets read in place"),
                "achieved": step_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": step_gbs / HBM_PEAK_GBS,
                "traffic": measured_traffic("step_" + w.name) if args.path == "cache" else None,
                "bytes_per_launch": f["step_bytes"], "us_per_launch": ms_per_step * 1e3,
                "what": "algorithmic bytes of one step (gather: every K/V row read and written once; each layer's "
                        "attention: every visible K/V row read once) over the step's wall time"}
    if f["pre_roofline"]["bound"] != "hbm":
        roofline["frac_of_floor"] = f["step_frac_of_floor"]   # compute-bound prefill: the floor is not bytes alone

    res = {
        "metric": "per-layer assemble+query-prefill us at 8K ctx",
        "value": ms_per_step * 1e3 / w.n_layers,
        "unit": "us/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: %d layers, Hq %d / Hkv %d, d %d, %d request(s), ctx %s, n_q %s"
                   % (w.name, w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, n_req,
                      ctx[:4], [rq.n_q for rq in w.requests[:4]]),
                   "layout": ("paged, %s block order" % args.block_order) if w.paged else "contiguous", "path": args.path,
                   "store": args.store, "pipelined": bool(pipelined), "shared_header": bool(args.shared_header),
                   "store_bytes_used": kvp.kvp_store_bytes_used(store)},
        "roofline": roofline,
        "roofline_attention": roofline_attention,
        "roofline_assemble": roofline_assemble if args.path == "cache" else None,
        "floor_us_per_layer": f["floor_us_per_layer"],
        "prefill": {"us_per_layer": f["pre_us"], "bytes_per_layer": f["pre_bytes"],
                    "flops_per_layer": f["pre_flops"], "achieved_GBs": f["pre_gbs"],
                    "hbm_frac": f["pre_gbs"] / HBM_PEAK_GBS, "achieved_TFLOPs": f["pre_tflops"],
                    "mfma_frac": f["pre_tflops"] / BF16_PEAK_TFLOPS},
        "assemble_us_per_layer": f["asm_us"] / w.n_layers,
        "step_us_per_layer": {"p50": float(np.percentile(step_ms, 50)) * 1e3 / w.n_layers,
                              "p99": float(np.percentile(step_ms, 99)) * 1e3 / w.n_layers,
                              "what": "per timed step, HIP events around assemble + all layers' prefill"},
    }
    if args.store == "host":
        # the packets cross PCIe at every assembly (or at every in-place read): that link bounds
        # the step; its rate is whole-step bytes read from the store over wall time
        store_bytes = (f["asm_bytes"] / 2.0) if args.path == "cache" else f["pre_bytes"] * w.n_layers
        res["roofline"] = {"bound": "pcie", "kernel": "reads of the host-resident store",
                           "achieved": store_bytes / (ms_per_step * 1e-3) / 1e9, "peak": PCIE_PEAK_GBS,
                           "unit": "GB/s", "frac": store_bytes / (ms_per_step * 1e-3) / 1e9 / PCIE_PEAK_GBS,
                           "traffic": None, "bytes_per_step": store_bytes}
    total_rows = sum(ctx) + tot_q
    res["tokens_per_s"] = total_rows / (ms_per_step * 1e-3)  # context + query positions per second
    res["query_tokens_per_s"] = tot_q / (ms_per_step * 1e-3)
    if n_req > 1 and args.per_request:
        res["per_request"] = per_request_latency(run, args, args.mixes)
    if not pipelined and args.store == "device" and not args.no_graph and not args.no_cpu_baseline:
        # The same step replayed from a HIP graph captured once: what a caller gains who captures
        # the launches of a repeated geometry (the per-layer launches of a short context are
        # launch-bound).  Reported beside `value`, which stays the eagerly launched step.
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            run["step"]()               # the plans of this geometry on this stream
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            try:
                with torch.cuda.graph(g, stream=side):
                    run["step"]()
                for _ in range(args.warmup):
                    g.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    g.replay()
                torch.cuda.synchronize()
                res["graph_replay"] = {"us_per_layer": (time.perf_counter() - t0) * 1e6 / args.steps / w.n_layers,
                                       "what": "the same step (every launch of it) replayed from a HIP graph captured once"}
            except Exception as e:      # (a call that cannot be captured says so; `value` does not depend on this)
                res["graph_replay"] = {"us_per_layer": None, "what": "not captured: %s" % e}
        note("graph replay done")
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, min(args.cpu_layers, w.n_layers))
        if not pipelined and args.store == "device":
            res["parity"] = parity(run, request=0, layer=w.n_layers - 1)
        note("cpu baseline and parity done")
    want_configs = args.configs == "all" or (args.configs == "auto" and args.workload == "llama_8k" and args.path == "cache"
                                             and args.store == "device" and not args.pipeline and not args.layers
                                             and not args.layout and not args.shared_header)
    if want_configs and not args.no_cpu_baseline:
        kvp.kvp_store_destroy(store)
        del run, store
        torch.cuda.empty_cache()
        cs, cw = args.config_steps, args.config_warmup
        res["configs"] = [
            config_record("tiny_fp32", args, cs, cw),                                   # config 1
            config_record("llama_k5", args, cs, cw),                                    # config 2
            config_record("qwen_k20", args, cs, cw),                                    # config 3
            config_record("llama_long_b8", args, cs, cw),                               # config 4 (4 layers instantiated)
            config_record("llama_long_b8_q32", args, cs, cw),                           # the same contexts, HBM-bound
            config_record("llama_long_b8_q1", args, cs, cw),                            # one decode step over them
            config_record("serving_mix", args, cs, cw, per_request=True),               # config 5 (1 layer, paged)
            config_record("llama_8k", args, cs, cw, path="packets"),                    # no cache: the store read in place
            config_record("llama_8k_pruned", args, cs, cw),                             # Sec. 5.4: compressed packets
            config_record("llama_8k_decode", args, cs, cw),                             # one generated token at 8K
        ]
        res["configs_note"] = ("short runs (%d steps after %d untimed) with only the retrieved packets stored; parity = "
                               "one request, first layer, against the CPU oracle" % (cs, cw))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
