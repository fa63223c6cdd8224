"""Runs a kvp_workloads.Workload through the HIP library (via the C ABI binding) and
through the CPU oracle, returning comparable numpy results.  Used by the GPU parity
tests and the smoke check."""
import numpy as np
import torch

import kvp_workloads as W
from kvp_setup import build_store, make_cache, needed_packets  # noqa: F401 (re-exported for the tests)


def _np(t):
    return W.to_numpy(t)


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def run_workload(w, layers=None, device="cuda:0", flags=0, block_order="random", store=None,
                 prerotate_with=None):
    """Full hot path on the GPU.  Returns dict(k, v, out, ctx): k[r], v[r] are numpy
    [n_layers][Hkv][ctx+n_q][d] logical caches (bf16 as uint16 bits) after the query append of
    the layers run; out[r][layer] float64 [n_q][Hq][d]."""
    import paper_2604_13226_amd as kvp
    layers = list(range(w.n_layers)) if layers is None else list(layers)
    own = store is None
    if own:
        store = build_store(w, kvp, device)
    cache = make_cache(w, kvp, store, device, block_order)
    n_req = len(w.requests)
    kvp.kvp_assemble(store, [(rq.packet_ids, rq.base_pos) for rq in w.requests], cache)
    ctx = [int(x) for x in cache.ctx_len[:n_req]]
    assert ctx == [w.ctx_len(r) for r in range(n_req)], (ctx,)
    q_off = np.zeros(n_req + 1, np.int32)
    for r in range(n_req):
        q_off[r + 1] = q_off[r] + w.requests[r].n_q
    tot_q = int(q_off[-1])
    max_ctx = max([ctx[r] + w.requests[r].n_q for r in range(n_req)] + [1])
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, n_req, tot_q, max_ctx), device)
    outs = [dict() for _ in range(n_req)]
    for layer in layers:
        qs, ks, vs = [], [], []
        for r in range(n_req):
            q, kn, vn = w.query(r, layer, device)
            if prerotate_with is not None:
                q, kn = prerotate_with(r, layer, q, kn, ctx[r])
            qs.append(q), ks.append(kn), vs.append(vn)
        q = torch.cat(qs) if qs else torch.empty(0)
        kn, vn = torch.cat(ks), torch.cat(vs)
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, layer, q.contiguous(), kn.contiguous(), vn.contiguous(),
                              q_off, ws, out, flags)
        torch.cuda.synchronize()
        for r in range(n_req):
            outs[r][layer] = _f64(out[q_off[r]:q_off[r + 1]])
    torch.cuda.synchronize()
    K, V = [], []
    for r in range(n_req):
        rows = ctx[r] + w.requests[r].n_q
        kl, vl = [], []
        for layer in range(w.n_layers):
            k, v = cache.logical(r, layer, rows)
            kl.append(_np(k)), vl.append(_np(v))
        K.append(np.stack(kl)), V.append(np.stack(vl))
    res = dict(k=K, v=V, out=outs, ctx=ctx, cache=cache, store=store)
    return res


def oracle_workload(w, layers=None, prerotated=False, prerotate_with=None, requests=None):
    """Same computation with the CPU oracle (contiguous logical caches).  `requests` limits
    the work to a sample of the requests (the other entries of the result are None)."""
    import oracle
    layers = list(range(w.n_layers)) if layers is None else list(layers)
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    npdt = np.float32 if w.dtype == "f32" else np.uint16
    K, V, outs, ctxs = [], [], [], []
    for r, rq in enumerate(w.requests):
        if requests is not None and r not in requests:
            K.append(None), V.append(None), outs.append(None), ctxs.append(w.ctx_len(r))
            continue
        pk, pv = [], []
        for p in rq.packet_ids:
            k, v = w.packet_kv(p)
            pk.append(_np(k)), pv.append(_np(v))
        rows = w.ctx_len(r) + rq.n_q
        shape = (w.n_layers, w.n_kv_heads, rows, w.head_dim)
        ko, vo = np.zeros(shape, npdt), np.zeros(shape, npdt)
        ko, vo, ctx = oracle.assemble(w.dtype, pk, pv, f, rq.base_pos, rows, ko, vo)
        o = {}
        for layer in layers:
            q, kn, vn = w.query(r, layer)
            if prerotate_with is not None:
                q, kn = prerotate_with(r, layer, q, kn, ctx)
            o[layer] = oracle.query_prefill(w.dtype, _np(q), _np(kn), _np(vn), f, ctx, ko[layer],
                                            vo[layer], prerotated)
        K.append(ko), V.append(vo), outs.append(o), ctxs.append(ctx)
    return dict(k=K, v=V, out=outs, ctx=ctxs)
