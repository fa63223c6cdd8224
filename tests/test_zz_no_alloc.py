"""kvp_query_prefill_static -- the entry point that allocates nothing -- against kvp_query_prefill
(same kernels: bit for bit) and against the CPU oracle (the attention tolerance), through the C
ABI, on two calls in a row of which the second is smaller, for both attention kernels."""
import numpy as np
import pytest
import torch

import kvp_workloads as W
from tests.gpu_harness import build_store, make_cache, oracle_workload

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def _inputs(w, layer, dev):
    parts = [w.query(r, layer, dev) for r in range(len(w.requests))]
    return tuple(torch.cat([p[i] for p in parts]).contiguous() for i in range(3))


def _run_both(w, kvp, store, dev):
    """One layer-0 call through each entry point on caches of their own.  Returns the two outputs,
    the two caches and the bytes of device memory that went missing across the static call."""
    n_req = len(w.requests)
    reqs = [(rq.packet_ids, rq.base_pos) for rq in w.requests]
    q_off = np.concatenate([[0], np.cumsum([rq.n_q for rq in w.requests])]).astype(np.int32)
    tot_q = int(q_off[-1])
    max_ctx = max(w.ctx_len(r) + w.requests[r].n_q for r in range(n_req))
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, n_req, tot_q, max_ctx), dev)
    q, kn, vn = _inputs(w, 0, dev)
    c_ref, c_new = make_cache(w, kvp, store, dev), make_cache(w, kvp, store, dev)
    kvp.kvp_assemble(store, reqs, c_ref)
    kvp.kvp_assemble(store, reqs, c_new)
    o_ref, o_new = torch.full_like(q, float("nan")), torch.full_like(q, float("nan"))
    kvp.kvp_query_prefill(store, c_ref, 0, q, kn, vn, q_off, ws, o_ref)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    kvp.kvp_query_prefill_static(store, c_new, 0, q, kn, vn, q_off, o_new)
    torch.cuda.synchronize()
    lost = free0 - torch.cuda.mem_get_info()[0]
    return o_ref, o_new, c_ref, c_new, lost


def _check(w, kvp, store, dev):
    o_ref, o_new, c_ref, c_new, lost = _run_both(w, kvp, store, dev)
    assert lost == 0, "device memory was allocated during the call: %d bytes" % lost
    assert not bool(torch.isnan(o_new.float()).any())
    assert torch.equal(o_new.view(torch.uint8), o_ref.view(torch.uint8)), "outputs differ from kvp_query_prefill's"
    assert torch.equal(c_new.k.view(torch.uint8), c_ref.k.view(torch.uint8))
    assert torch.equal(c_new.v.view(torch.uint8), c_ref.v.view(torch.uint8))
    ref = oracle_workload(w, layers=[0])
    off = 0
    for r, rq in enumerate(w.requests):
        got = o_new[off:off + rq.n_q].float().cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(got - ref["out"][r][0]))) if rq.n_q else 0.0
        assert err <= TOL[w.dtype], (w.name, r, err)
        rows = w.ctx_len(r) + rq.n_q
        k, v = c_new.logical(r, 0, rows)
        assert np.array_equal(W.to_numpy(k), ref["k"][r][0]) and np.array_equal(W.to_numpy(v), ref["v"][r][0])
        off += rq.n_q


@pytest.mark.parametrize("kind", ["bf16 mfma", "f32 generic"])
def test_two_calls_in_a_row_the_second_smaller(gpu_device, kind):
    import paper_2604_13226_amd as kvp
    dev = "cuda:0"
    if kind == "bf16 mfma":
        big = W.llama_k5(n_layers=1, n_packets=8)                     # ~3K rows, 32 query rows, split-KV
        small = W.llama_k5(n_layers=1, n_packets=8)
        small.requests = [W.Request(big.requests[0].packet_ids[:2], 7)]
    else:
        big = W.random_small(31, dtype="f32", d=64, n_q_heads=4, n_kv_heads=2, n_layers=1, n_packets=6, k=5,
                             n_q=9, max_len=400)
        small = W.random_small(31, dtype="f32", d=64, n_q_heads=4, n_kv_heads=2, n_layers=1, n_packets=6, k=5,
                               n_q=9, max_len=400)
        small.requests = [W.Request(big.requests[0].packet_ids[:1], 3)]
    store = build_store(big, kvp, dev)
    assert kvp.kvp_static_workspace_bytes() == (31 << 20)
    _check(big, kvp, store, dev)
    _check(small, kvp, store, dev)       # the scratch still holds the larger call's plan and partial results
    _check(big, kvp, store, dev)         # and back: the plan is replaced again
    kvp.kvp_store_destroy(store)


def test_sizes_beyond_the_scratch_are_rejected(gpu_device):
    import paper_2604_13226_amd as kvp
    dev = "cuda:0"
    import os
    w = W.llama_long_b8(n_layers=1, n_packets=16, batch=16, k=2, n_q=128)
    # (the planner's own split counts keep the partial rows of any call under the scratch's size; a
    # finer cut than it would choose -- 4 kv ranges for each of 256 row blocks: 1024 slots of 256
    # fp16 rows, 69 MB -- does not fit)
    os.environ["KVP_ATTN_TARGET_ITEMS"] = "1024"
    try:
        store = build_store(w, kvp, dev)
    finally:
        del os.environ["KVP_ATTN_TARGET_ITEMS"]
    cache = make_cache(w, kvp, store, dev)
    reqs = [(rq.packet_ids, rq.base_pos) for rq in w.requests]
    kvp.kvp_assemble(store, reqs, cache)
    q_off = np.arange(17, dtype=np.int32) * 128
    q, kn, vn = _inputs(w, 0, dev)
    out = torch.full_like(q, 5.0)
    k_before = cache.k.clone()
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_query_prefill_static(store, cache, 0, q, kn, vn, q_off, out)
    assert e.value.code == kvp.KVP_E_CAPACITY and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 5.0).all()) and torch.equal(cache.k, k_before)      # nothing was launched
    # the same call fits a caller workspace
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 16, 2048, 1056 + 128), dev)
    kvp.kvp_query_prefill(store, cache, 0, q, kn, vn, q_off, ws, out)
    torch.cuda.synchronize()
    assert not bool((out == 5.0).all())
    kvp.kvp_store_destroy(store)
