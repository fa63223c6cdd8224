"""Sets a kvp_workloads.Workload up on the GPU through the library's binding: the packet store
and a cache of the workload's layout.  Used by the benchmark, the smoke check and the GPU tests.
Input plumbing only: it holds none of the method's arithmetic and knows nothing of the oracle."""
import numpy as np
import torch


def needed_packets(w):
    return sorted({p for rq in w.requests for p in rq.packet_ids})


def build_store(w, kvp, device="cuda:0", packets=None, max_positions=None, extra_bytes=0, arena="device",
                progress=None):
    packets = needed_packets(w) if packets is None else packets
    arena_bytes = sum(kvp.packet_bytes(w.n_layers, w.n_kv_heads, w.head_dim, w.dtype, int(w.packet_lens[p]))
                      for p in packets) + extra_bytes
    if w.shared_header:
        arena_bytes += kvp.packet_bytes(w.n_layers, w.n_kv_heads, w.head_dim, w.dtype, w.n_header)
    if max_positions is None:
        max_positions = max([w.ctx_len(r) + w.requests[r].n_q for r in range(len(w.requests))] + [1]) + 64
    store = kvp.kvp_store_create(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype,
                                 w.rope_base, max_positions, max(arena_bytes, 256), w.n_header,
                                 w.n_trailer, device=0, arena=arena)
    if w.shared_header:
        kvp.kvp_store_put_header(store, *w.header_kv(device))
    for i, p in enumerate(packets):
        k, v = w.packet_kv(p, device=device)
        if w.shared_header and k.shape[2] > w.n_header:    # the header rows are in the store already
            kvp.kvp_store_put_body(store, p, k[:, :, w.n_header:].contiguous(), v[:, :, w.n_header:].contiguous())
        elif w.prune is None:
            kvp.kvp_store_put(store, p, k, v)
        else:
            keep = [torch.as_tensor(w.kept_rows(p, l), device=device) for l in range(w.n_layers)]
            kvp.kvp_store_put_compressed(store, p, int(w.packet_lens[p]),
                                         [k[l][:, keep[l]].contiguous() for l in range(w.n_layers)],
                                         [v[l][:, keep[l]].contiguous() for l in range(w.n_layers)])
        if progress is not None and i % 32 == 31:
            progress(i + 1, len(packets))
    torch.cuda.synchronize()
    return store


def make_cache(w, kvp, store, device="cuda:0", block_order="random", t_slack=5):
    n_req = len(w.requests)
    rows = [w.ctx_len(r) + w.requests[r].n_q for r in range(n_req)]
    if not w.paged:
        c = kvp.Cache.contiguous(store, n_req, max(rows + [1]) + t_slack, device)
        return c.with_ctx_rows(w.n_layers) if w.prune is not None else c
    bs = w.block_size
    nblk = [(x + bs - 1) // bs for x in rows]
    total = sum(nblk) + 3
    rng = np.random.default_rng(w.seed + 77)
    pool = rng.permutation(total) if block_order == "random" else np.arange(total)
    table = np.zeros((n_req, max(nblk + [1])), np.int32)
    at = 0
    for r in range(n_req):
        table[r, :nblk[r]] = pool[at:at + nblk[r]]
        at += nblk[r]
    c = kvp.Cache.paged(store, n_req, total, table, bs, device)
    return c.with_ctx_rows(w.n_layers) if w.prune is not None else c
