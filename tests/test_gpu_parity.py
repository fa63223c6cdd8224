"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Assembly (and the appended query K/V) must match bit for bit; attention
within 1e-5 (fp32 path) / 2e-2 (bf16 inputs, fp32 accumulation) max abs error."""
import os

import numpy as np
import pytest
import torch

import kvp_workloads as W
from tests.gpu_harness import build_store, make_cache, oracle_workload, run_workload

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
# Second bar, on the root-mean-square error relative to the root-mean-square output.  The
# bf16 path rounds Q (after rotation and scaling), P and the output to 8 significant bits,
# each a relative error of at most 2^-9 with no preferred sign; a systematic slip of a few
# per cent (a wrong normaliser, a reference maximum that differs between lanes of one row)
# stays under the absolute bar on outputs of size 0.05 but not under this one.
REL_RMS_TOL = {"f32": 2e-6, "bf16": 6e-3}
WORST_REL_RMS = {"f32": 0.0, "bf16": 0.0}


def check_output(o, ref, dtype, tag):
    """Both bars for one request-layer output; returns the maximum absolute error."""
    assert np.all(np.isfinite(o)), ("non-finite output",) + tuple(tag)
    err = float(np.max(np.abs(o - ref)))
    assert err <= TOL[dtype], tuple(tag) + (err,)
    rms_ref = float(np.sqrt(np.mean(ref * ref)))
    if rms_ref > 0:
        rel = float(np.sqrt(np.mean((o - ref) ** 2))) / rms_ref
        WORST_REL_RMS[dtype] = max(WORST_REL_RMS[dtype], rel)
        assert rel <= REL_RMS_TOL[dtype], tuple(tag) + ("relative rms", rel)
    return err


def compare(w, got, ref, layers=None):
    layers = range(w.n_layers) if layers is None else layers
    worst = 0.0
    for r in range(len(w.requests)):
        assert got["ctx"][r] == ref["ctx"][r]
        for layer in layers:
            assert np.array_equal(got["k"][r][layer], ref["k"][r][layer]), (w.name, "K", r, layer)
            assert np.array_equal(got["v"][r][layer], ref["v"][r][layer]), (w.name, "V", r, layer)
            if w.requests[r].n_q == 0:
                continue
            worst = max(worst, check_output(got["out"][r][layer], ref["out"][r][layer], w.dtype, (w.name, r, layer)))
    return worst


def test_config1_tiny_fp32(gpu_device):
    w = W.tiny_fp32()
    err = compare(w, run_workload(w), oracle_workload(w))
    print("tiny_fp32 max abs err", err)


@pytest.mark.parametrize("case", [
    dict(seed=11, d=2, n_q_heads=1, n_kv_heads=1, k=1, n_q=1, max_len=1),
    dict(seed=12, d=8, n_q_heads=4, n_kv_heads=2, k=3, n_q=5),
    dict(seed=13, d=8, n_q_heads=7, n_kv_heads=1, k=3, n_q=5, n_req=3),
    dict(seed=14, d=16, n_q_heads=4, n_kv_heads=2, k=0, n_q=6),
    dict(seed=15, d=24, n_q_heads=4, n_kv_heads=2, k=3, n_q=3, base_pos=11),
    dict(seed=16, d=64, n_q_heads=14, n_kv_heads=2, k=6, n_q=9, max_len=150, n_packets=4),
    dict(seed=17, d=256, n_q_heads=2, n_kv_heads=2, k=2, n_q=3, max_len=70),
])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_ragged_shapes(gpu_device, case, dtype):
    w = W.random_small(dtype=dtype, **case)
    compare(w, run_workload(w), oracle_workload(w))


def _random_geometry(seed):
    """A seeded random batch: 1-4 requests, ragged packets, ragged (some empty) queries, head
    groupings 1 / 4 / 7, every head dim the vector gather takes, either dtype and layout, with or
    without the shared header, sometimes a caller prefix below base_pos."""
    rng = np.random.default_rng(seed)
    dtype = "bf16" if rng.random() < 0.6 else "f32"
    d = int(rng.choice([64, 128, 128, 128, 128, 256])) if dtype == "bf16" else int(rng.choice([8, 64, 128]))
    n_kv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 4, 7]))
    n_req = int(rng.integers(1, 5))
    n_packets = int(rng.integers(2, 7))
    big = dtype == "bf16" and d == 128 and rng.random() < 0.75          # the MFMA kernel with several row blocks
    w = W.random_small(seed, dtype=dtype, d=d, n_q_heads=n_kv * g, n_kv_heads=n_kv, n_layers=int(rng.integers(1, 3)),
                       n_packets=n_packets, k=1, n_q=1, max_len=int(rng.choice([9, 70, 300])), n_req=n_req)
    for rq in w.requests:
        rq.packet_ids = [int(x) for x in rng.integers(0, n_packets, size=int(rng.integers(0, 6)))]
        rq.n_q = int(rng.integers(0, 150 if big else 12))
        rq.base_pos = int(rng.integers(0, 40)) if rng.random() < 0.3 else 0
    if all(rq.n_q == 0 for rq in w.requests):
        w.requests[0].n_q = 3
    w.paged = bool(rng.random() < 0.4)
    w.block_size = int(rng.choice([16, 32, 64])) if big or dtype == "bf16" else int(rng.choice([4, 16]))
    if rng.random() < 0.3:
        w.n_header, w.shared_header = int(rng.choice([1, 4, 8])), True
    return w


@pytest.mark.parametrize("seed", range(300, 340))
def test_random_geometries(gpu_device, seed):
    w = _random_geometry(seed)
    compare(w, run_workload(w), oracle_workload(w))


@pytest.mark.parametrize("seed", range(700, 748))
def test_random_geometries_with_random_launch_shapes(gpu_device, seed):
    """The same random batches with the planner's choices overridden at random: how finely
    split-KV cuts, the row block, the two-group workgroup shape, half blocks on or off, the
    gather's tile rows and whether its workgroups move K and V together, the streaming hint of the
    tile loads and the generic kernel.  Results must not depend on any of them."""
    rng = np.random.default_rng(seed + 10000)
    w = _random_geometry(seed)
    env = {"KVP_ATTN_TARGET_ITEMS": str(int(rng.choice([1, 7, 64, 300, 4000]))),
           "KVP_ASM_TILE_ROWS": str(int(rng.choice([16, 32, 64])))}
    if rng.random() < 0.5:
        env["KVP_ATTN_BM"] = str(int(rng.choice([128, 256])))
    if rng.random() < 0.5:
        env["KVP_ATTN_SPLIT_IN_WG"] = str(int(rng.integers(0, 2)))
    if rng.random() < 0.3:
        env["KVP_ATTN_MIXED"] = "0"
    if rng.random() < 0.15:
        env["KVP_FORCE_GENERIC_ATTENTION"] = "1"
    if rng.random() < 0.2:
        env["KVP_ASM_NONTEMPORAL"] = "1"
    if rng.random() < 0.2:
        env["KVP_PLAN_COPY_ENGINE"] = "1"
    if rng.random() < 0.4:
        env["KVP_ATTN_NT_LOADS"] = str(int(rng.integers(0, 2)))
    if rng.random() < 0.4:
        env["KVP_ASM_SPLIT_KV"] = "0"
    os.environ.update(env)
    try:
        got = run_workload(w)
    finally:
        for k in env:
            os.environ.pop(k, None)
    try:
        compare(w, got, oracle_workload(w))
    except AssertionError as e:
        raise AssertionError("with %s: %s" % (env, e))


@pytest.mark.parametrize("mk", [
    lambda: W.llama_k5(n_layers=2, n_packets=16),
    lambda: W.qwen_k20(n_layers=2, n_packets=40),
    lambda: W.llama_8k(n_layers=1, n_packets=16),
])
def test_model_shapes_reduced_depth(gpu_device, mk):
    w = mk()
    err = compare(w, run_workload(w), oracle_workload(w))
    print(w.name, "max abs err", err)


def test_batch_with_shared_packets(gpu_device):
    # several requests, the same packet in more than one of them and twice in one
    w = W.llama_long_b8(n_layers=1, n_packets=6, batch=3, k=4, n_q=40)
    w.requests[1].packet_ids = [2, 2, 5, 2]
    w.requests[2].n_q = 0
    compare(w, run_workload(w), oracle_workload(w))


@pytest.mark.parametrize("order", ["random", "sequential"])
def test_paged_serving_mix_small(gpu_device, order):
    w = W.serving_mix(n_packets=64, n_req=6)
    for rq in w.requests:
        rq.packet_ids = rq.packet_ids[:4]
        rq.n_q = min(rq.n_q, 70)
    got = run_workload(w, block_order=order)
    compare(w, got, oracle_workload(w))


def test_paged_fp32_small_blocks(gpu_device):
    w = W.random_small(31, dtype="f32", d=64, k=5, n_q=7, max_len=40, n_req=2, n_packets=6)
    w.paged, w.block_size = True, 4
    compare(w, run_workload(w), oracle_workload(w))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prerotated_flag(gpu_device, dtype):
    import oracle
    import paper_2604_13226_amd as kvp
    w = W.random_small(41, dtype=dtype, d=64, k=3, n_q=6, max_len=50, n_layers=1)
    f = oracle.inv_freq(w.rope_base, w.head_dim)

    def prerot(r, layer, q, kn, ctx):
        # the caller's own rotation: oracle arithmetic on the CPU, then back to the device
        dev = q.device
        qn, knn = W.to_numpy(q), W.to_numpy(kn)
        if dtype == "bf16":
            widen = lambda a: (a.astype(np.uint32) << 16).view(np.float32)
        else:
            widen = lambda a: a
        def rot(a):
            a = widen(a)
            out = np.empty_like(a)
            for t in range(a.shape[0]):
                for h in range(a.shape[1]):
                    out[t, h] = oracle.rotate(np.ascontiguousarray(a[t, h]), ctx + t, f)
            return torch.from_numpy(out).to(w.torch_dtype).to(dev)
        return rot(qn), rot(knn)

    got = run_workload(w, flags=kvp.KVP_PREROTATED, prerotate_with=prerot)
    ref = oracle_workload(w, prerotated=True, prerotate_with=prerot)
    compare(w, got, ref)


def test_special_values_bit_exact(gpu_device):
    """Denormals, signed zeros, large magnitudes and rounding ties go through the same
    arithmetic on both sides."""
    import oracle
    import paper_2604_13226_amd as kvp
    rng = np.random.default_rng(5)
    n_layers, n_kv, d = 1, 2, 128
    lens = [3, 70, 64]
    pk, pv = [], []
    for n in lens:
        bits = rng.integers(0, 1 << 16, size=(n_layers, n_kv, n, d), dtype=np.uint16)
        exp = (bits >> 7) & 0xFF
        bits[exp == 0xFF] &= 0x807F                      # no inf / nan: make them denormals
        big = exp >= 0xF0
        bits[big] = (bits[big] & 0x807F) | (0x7E << 7)   # keep products finite
        bits[0, 0, 0, :8] = [0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x3F80, 0xBF80]
        pk.append(bits)
        pv.append(rng.integers(0, 1 << 16, size=(n_layers, n_kv, n, d), dtype=np.uint16))
    f = oracle.inv_freq(5.0e5, d)
    ko, vo, ctx = oracle.assemble("bf16", pk, pv, f, 0, sum(lens))
    store = kvp.kvp_store_create(n_layers, 8, n_kv, d, "bf16", 5.0e5, 1024, 1 << 22)
    for i, (a, b) in enumerate(zip(pk, pv)):
        ta = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
        tb = torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)
        kvp.kvp_store_put(store, i, ta, tb)              # host source
    cache = kvp.Cache.contiguous(store, 1, sum(lens))
    kvp.kvp_assemble(store, [([0, 1, 2], 0)], cache)
    torch.cuda.synchronize()
    k, v = cache.logical(0, 0, ctx)
    assert np.array_equal(W.to_numpy(k), ko[0])
    assert np.array_equal(W.to_numpy(v), vo[0])


def test_layer_range_and_untouched_rows(gpu_device):
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=3, n_packets=8)
    w.requests[0].packet_ids = w.requests[0].packet_ids[:2]
    w.requests[0].base_pos = 5
    store = build_store(w, kvp)
    cache = make_cache(w, kvp, store, t_slack=9)
    cache.k.fill_(7.0)
    cache.v.fill_(7.0)
    kvp.kvp_assemble(store, [(w.requests[0].packet_ids, 5)], cache, layer_begin=1, layer_end=2)
    torch.cuda.synchronize()
    ctx = int(cache.ctx_len[0])
    ref = oracle_workload(w, layers=[])
    for layer in range(3):
        k = W.to_numpy(cache.k[0, layer])
        v = W.to_numpy(cache.v[0, layer])
        seven = W.to_numpy(torch.tensor([7.0], dtype=torch.bfloat16))[0]
        if layer == 1:
            assert np.array_equal(k[:, 5:ctx], ref["k"][0][1][:, 5:ctx])
            assert np.array_equal(v[:, 5:ctx], ref["v"][0][1][:, 5:ctx])
            assert np.all(k[:, :5] == seven) and np.all(k[:, ctx:] == seven)
            assert np.all(v[:, :5] == seven) and np.all(v[:, ctx:] == seven)
        else:
            assert np.all(k == seven) and np.all(v == seven)


def test_failed_calls_change_nothing_on_device(gpu_device):
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=1, n_packets=8)
    store = build_store(w, kvp)
    cache = kvp.Cache.contiguous(store, 1, 100)              # far too small
    cache.k.fill_(3.0)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(store, [(w.requests[0].packet_ids, 0)], cache)
    assert e.value.code == kvp.KVP_E_CAPACITY
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(store, [([123456], 0)], cache)
    assert e.value.code == kvp.KVP_E_NOTFOUND
    torch.cuda.synchronize()
    assert bool((cache.k == 3.0).all())
    ws = kvp.alloc_workspace(256)
    q = torch.zeros(4, 32, 128, dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros(4, 8, 128, dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 9.0)
    big = kvp.Cache.contiguous(store, 1, 4096)               # a context long enough to be split: partial rows need a workspace
    big.k.fill_(3.0)
    big.ctx_len[0] = 3000
    with pytest.raises(kvp.KvpError) as e:                   # workspace too small
        kvp.kvp_query_prefill(store, big, 0, q, kn, kn, [0, 4], ws, out)
    assert e.value.code == kvp.KVP_E_CAPACITY
    torch.cuda.synchronize()
    assert bool((out == 9.0).all()) and bool((big.k == 3.0).all()) and bool((cache.k == 3.0).all())


def test_a_failed_prefill_call_keeps_the_kept_plans(gpu_device):
    """A call with a new geometry that fails on its workspace must not evict a kept plan: the
    geometries run before it are still found (a hit plans nothing, so the plan the store last
    built stays the one of the last miss)."""
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=1, n_packets=8)
    store = build_store(w, kvp)
    cache = kvp.Cache.contiguous(store, 1, 6000)
    q = torch.zeros(4, 32, 128, dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros(4, 8, 128, dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, 4, 6000))
    geoms = [300 + 64 * i for i in range(8)]                 # as many as the store keeps (max(8, n_layers + 1))
    for c in geoms:
        cache.ctx_len[0] = c
        kvp.kvp_query_prefill(store, cache, 0, q, kn, kn, [0, 4], ws, out)
    last = kvp.kvp_debug_last_plan(store, 1).copy()
    cache.ctx_len[0] = 5000
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_query_prefill(store, cache, 0, q, kn, kn, [0, 4], kvp.alloc_workspace(256), out)
    assert e.value.code == kvp.KVP_E_CAPACITY
    for c in geoms:
        cache.ctx_len[0] = c
        kvp.kvp_query_prefill(store, cache, 0, q, kn, kn, [0, 4], ws, out)
        assert np.array_equal(kvp.kvp_debug_last_plan(store, 1), last), c
    torch.cuda.synchronize()


def test_split_invariance(gpu_device):
    """The split-KV reduction is exact algebra: any number of splits gives the same result
    within tolerance, including splits that see no visible row."""
    w = W.llama_k5(n_layers=1, n_packets=8)
    ref = oracle_workload(w)
    for target in ("1", "16", "200", "4000"):
        os.environ["KVP_ATTN_TARGET_ITEMS"] = target
        try:
            got = run_workload(w)
        finally:
            del os.environ["KVP_ATTN_TARGET_ITEMS"]
        compare(w, got, ref)


@pytest.mark.parametrize("k", [60, -60, 0])
def test_values_scaled_by_a_power_of_two_scale_the_output(gpu_device, k):
    """The split-KV partial rows are fp16 scaled per row by a power of two chosen from the row's
    largest magnitude.  Scaling every value row (V and V_new) by 2^k scales every product and sum of
    the path exactly, so the output must be the unscaled output times 2^k, whatever the magnitude:
    2^60 and 2^-60 are far outside what fp16 holds without the per-row exponent.  Bit for bit but
    for the merge weights: a partial row's reference travels as the float m + e, whose rounding
    depends on e's size (relative 2^-17 at most), which may move an output by one bf16 step."""
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=1, n_packets=8)
    n_q = w.requests[0].n_q
    outs = []
    for scale in (1.0, 2.0 ** k):
        store = kvp.kvp_store_create(1, w.n_q_heads, w.n_kv_heads, w.head_dim, "bf16", w.rope_base, 4096,
                                     sum(kvp.packet_bytes(1, w.n_kv_heads, w.head_dim, "bf16", int(w.packet_lens[p]))
                                         for p in w.requests[0].packet_ids), 8, 8, device=0)
        for p in w.requests[0].packet_ids:
            kk, vv = w.packet_kv(p, device="cuda")
            kvp.kvp_store_put(store, p, kk, (vv.float() * scale).to(torch.bfloat16))
        cache = make_cache(w, kvp, store)
        kvp.kvp_assemble(store, [(w.requests[0].packet_ids, 0)], cache)
        q, kn, vn = w.query(0, 0, "cuda")
        vn = (vn.float() * scale).to(torch.bfloat16)
        ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, n_q, w.ctx_len(0) + n_q))
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, 0, q, kn, vn, [0, n_q], ws, out)
        torch.cuda.synchronize()
        assert int(kvp.kvp_debug_last_plan(store, 1)[4]) > 0          # the call was split: partial rows were used
        outs.append(out.float().cpu().numpy().astype(np.float64))
    assert np.all(np.isfinite(outs[1]))
    want, got = outs[0], outs[1] / 2.0 ** k
    rowmax = np.abs(want).max(axis=-1, keepdims=True)
    assert np.all(np.abs(got - want) <= 2.0 ** -7 * np.abs(want) + 2.0 ** -11 * rowmax)   # one bf16 step; tiny elements: the fp16 rows' step
    assert np.mean(got == want) > 0.99
    if k == 0:
        assert np.array_equal(got, want)


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("target", [None, "3000"])
def test_half_blocks_in_a_launch_of_256_row_blocks(gpu_device, paged, target):
    """A request with 4 n_q >= 256 packed rows makes the launch use 256-row blocks; groups of at
    most 128 rows (the last rows of a request, or a whole small request) then run as half blocks
    inside the same launch -- unsplit and, with many work items asked for, split over KV with
    partial slots of the launch's 256-row layout."""
    w = W.llama_long_b8(n_layers=1, n_packets=6, batch=4, k=3, n_q=89)      # 356 rows: 256 + 100
    w.packet_lens[:] = [700, 130, 64, 529, 300, 63]
    w.requests[1].n_q = 114                                                # 456 rows: 256 + 200 (a full block)
    w.requests[2].n_q = 20                                                 # 80 rows: one half block
    w.requests[3].n_q = 64                                                 # 256 rows exactly
    w.paged = paged
    if target:
        os.environ["KVP_ATTN_TARGET_ITEMS"] = target
    try:
        got = run_workload(w)
    finally:
        os.environ.pop("KVP_ATTN_TARGET_ITEMS", None)
    import paper_2604_13226_amd as kvp
    plan = kvp.kvp_debug_last_plan(got["store"], 1)
    assert plan[1] == 256                                                   # the launch's row block
    compare(w, got, oracle_workload(w))


@pytest.mark.parametrize("dtype,d,ctx_rows", [("f32", 8, 600), ("f32", 2, 300), ("bf16", 64, 1300), ("f32", 24, 700),
                                              ("bf16", 256, 900)])
def test_many_splits_with_small_head_dims(gpu_device, dtype, d, ctx_rows):
    """More kv ranges per group than a row has 16-byte chunks (or columns): the merge of the
    splits hands the weights around by lane shuffles, which must not depend on how many lanes
    a row of head_dim d keeps busy."""
    w = W.random_small(71, dtype=dtype, d=d, n_q_heads=4, n_kv_heads=2, n_layers=1, n_packets=3, k=3, n_q=5, max_len=9)
    w.packet_lens[:] = [ctx_rows // 2, ctx_rows // 3, ctx_rows - ctx_rows // 2 - ctx_rows // 3]
    w.requests[0].packet_ids = [0, 1, 2]
    os.environ["KVP_ATTN_TARGET_ITEMS"] = "4000"
    try:
        got = run_workload(w)
    finally:
        os.environ.pop("KVP_ATTN_TARGET_ITEMS", None)
    import paper_2604_13226_amd as kvp
    plan = kvp.kvp_debug_last_plan(got["store"], 1)
    groups = plan[6:6 + 6 * int(plan[2])].reshape(int(plan[2]), 6)
    assert groups[:, 5].max() == (ctx_rows + 5 + 63) // 64 > 4              # one range per 64 rows
    compare(w, got, oracle_workload(w))


def test_long_query_without_packets(gpu_device):
    """No cached context at all (the baseline without packets) and 1500 query tokens: plain
    causal self-attention over 24 tiles of query rows, 6000 packed rows per kv head."""
    w = W.llama_long_b8(n_layers=1, n_packets=2, batch=2, k=1, n_q=1500)
    w.n_q_heads, w.n_kv_heads = 8, 2
    w.packet_lens[:] = [70, 64]
    w.requests[0].packet_ids = []
    w.requests[1].packet_ids = [1, 0]
    w.requests[1].n_q = 700
    compare(w, run_workload(w), oracle_workload(w))


def test_side_stream_and_two_stores(gpu_device):
    """The whole path on a stream other than the current one, with a second store of another
    shape used in between (plans and their buffers belong to the store and the stream)."""
    import paper_2604_13226_amd as kvp
    wa = W.llama_k5(n_layers=2, n_packets=8)
    wb = W.qwen_k20(n_layers=1, n_packets=24)
    refs = [oracle_workload(wa), oracle_workload(wb)]
    side = torch.cuda.Stream()
    stores = [build_store(w, kvp) for w in (wa, wb)]
    caches = [make_cache(w, kvp, st) for w, st in zip((wa, wb), stores)]
    torch.cuda.synchronize()
    outs = [dict(), dict()]
    with torch.cuda.stream(side):
        for i, (w, st, c) in enumerate(zip((wa, wb), stores, caches)):
            kvp.kvp_assemble(st, [(rq.packet_ids, rq.base_pos) for rq in w.requests], c, stream=side)
        wss = [kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(st, 1, w.requests[0].n_q, w.ctx_len(0) + w.requests[0].n_q))
               for w, st in zip((wa, wb), stores)]
        for layer in range(2):
            for i, (w, st, c) in enumerate(zip((wa, wb), stores, caches)):      # the two stores take turns
                if layer >= w.n_layers:
                    continue
                q, kn, vn = w.query(0, layer, "cuda")
                out = torch.full_like(q, float("nan"))
                kvp.kvp_query_prefill(st, c, layer, q, kn, vn, [0, w.requests[0].n_q], wss[i], out, stream=side)
                outs[i][layer] = out
    side.synchronize()
    for i, w in enumerate((wa, wb)):
        rows = w.ctx_len(0) + w.requests[0].n_q
        for layer in range(w.n_layers):
            k, v = caches[i].logical(0, layer, rows)
            assert np.array_equal(W.to_numpy(k), refs[i]["k"][0][layer]), (w.name, layer, "K")
            assert np.array_equal(W.to_numpy(v), refs[i]["v"][0][layer]), (w.name, layer, "V")
            check_output(outs[i][layer].float().cpu().numpy().astype(np.float64), refs[i]["out"][0][layer], w.dtype,
                         (w.name, "side stream", layer))
    for st in stores:
        kvp.kvp_store_destroy(st)


def test_generic_kernel_on_bf16_model_shape(gpu_device):
    w = W.llama_k5(n_layers=1, n_packets=8)
    w.requests[0].packet_ids = w.requests[0].packet_ids[:2]
    os.environ["KVP_FORCE_GENERIC_ATTENTION"] = "1"
    try:
        got = run_workload(w)
    finally:
        del os.environ["KVP_FORCE_GENERIC_ATTENTION"]
    compare(w, got, oracle_workload(w))


def test_full_size_llama_k5_sampled(gpu_device):
    """Config 2 at full depth (32 layers, the launch configuration the benchmark times):
    assembly bit-exact on every layer, attention on sampled layers."""
    w = W.llama_k5()
    layers = [0, 13, 31]
    got = run_workload(w, layers=layers)
    ref = oracle_workload(w, layers=layers)
    r = 0
    ctx = ref["ctx"][0]
    for layer in range(w.n_layers):
        rows = ctx if layer not in layers else ctx + w.requests[0].n_q
        assert np.array_equal(got["k"][r][layer][:, :rows], ref["k"][r][layer][:, :rows]), layer
        assert np.array_equal(got["v"][r][layer][:, :rows], ref["v"][r][layer][:, :rows]), layer
    for layer in layers:
        check_output(got["out"][r][layer], ref["out"][r][layer], w.dtype, (w.name, layer))


def test_full_size_qwen_k20_sampled(gpu_device):
    """Config 3 at full depth (28 layers, 4 KV heads, 20 packets, 448 packed rows per KV head:
    two row blocks of 256, the second three quarters full), as the benchmark launches it:
    assembly bit-exact on every layer, attention on sampled layers."""
    w = W.qwen_k20()
    layers = [0, 9, 27]
    got = run_workload(w, layers=layers)
    ref = oracle_workload(w, layers=layers)
    r = 0
    ctx = ref["ctx"][0]
    for layer in range(w.n_layers):
        rows = ctx if layer not in layers else ctx + w.requests[0].n_q
        assert np.array_equal(got["k"][r][layer][:, :rows], ref["k"][r][layer][:, :rows]), layer
        assert np.array_equal(got["v"][r][layer][:, :rows], ref["v"][r][layer][:, :rows]), layer
    for layer in layers:
        check_output(got["out"][r][layer], ref["out"][r][layer], w.dtype, (w.name, layer))


@pytest.mark.parametrize("mk", [lambda: W.tiny_fp32(), lambda: W.llama_k5(n_layers=1, n_packets=8)])
def test_decode_steps_after_prefill(gpu_device, mk):
    """After the query prefill the caller advances ctx_len by n_q; every later token is one
    more kvp_query_prefill with a single query row (auto-regressive decoding over the composed
    cache, Sec. 3.1).  Appended rows stay bit-exact, outputs stay within tolerance."""
    import oracle
    import paper_2604_13226_amd as kvp
    w = mk()
    w.requests[0].packet_ids = w.requests[0].packet_ids[:2]
    steps = 3
    rq = w.requests[0]
    store = build_store(w, kvp, max_positions=w.ctx_len(0) + rq.n_q + steps + 8)
    cache = kvp.Cache.contiguous(store, 1, w.ctx_len(0) + rq.n_q + steps)
    kvp.kvp_assemble(store, [(rq.packet_ids, 0)], cache)
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, rq.n_q, w.ctx_len(0) + rq.n_q + steps))
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    pk = [W.to_numpy(w.packet_kv(p)[0]) for p in rq.packet_ids]
    pv = [W.to_numpy(w.packet_kv(p)[1]) for p in rq.packet_ids]
    rows = w.ctx_len(0) + rq.n_q + steps
    npdt = np.float32 if w.dtype == "f32" else np.uint16
    ko = np.zeros((w.n_layers, w.n_kv_heads, rows, w.head_dim), npdt)
    vo = np.zeros_like(ko)
    ko, vo, ctx = oracle.assemble(w.dtype, pk, pv, f, 0, rows, ko, vo)
    n_q = rq.n_q
    for step in range(steps + 1):
        q, kn, vn = (W.normal_tensor((n_q, h, w.head_dim), w.seed, 40 + i, step, 1.0 if i == 0 else w.kv_scale,
                                     w.torch_dtype, "cuda")
                     for i, h in enumerate((w.n_q_heads, w.n_kv_heads, w.n_kv_heads)))
        out = torch.empty_like(q)
        assert int(cache.ctx_len[0]) == ctx
        kvp.kvp_query_prefill(store, cache, 0, q, kn, vn, [0, n_q], ws, out)
        torch.cuda.synchronize()
        ref = oracle.query_prefill(w.dtype, W.to_numpy(q), W.to_numpy(kn), W.to_numpy(vn), f, ctx, ko[0], vo[0])
        check_output(out.float().cpu().numpy().astype(np.float64), ref, w.dtype, ("decode step", step))
        ctx += n_q
        cache.ctx_len[0] = ctx            # the caller advances the context after the layer(s)
        k, v = cache.logical(0, 0, ctx)
        assert np.array_equal(W.to_numpy(k), ko[0][:, :ctx]) and np.array_equal(W.to_numpy(v), vo[0][:, :ctx])
        n_q = 1


def _run_packets(w, layers, flags=0, prerotate_with=None, arena="device"):
    """kvp_prefill_packets over the workload: returns (out[r][layer], k_tail[r][layer])."""
    import paper_2604_13226_amd as kvp
    store = build_store(w, kvp, arena=arena)
    n_req = len(w.requests)
    q_off = np.zeros(n_req + 1, np.int32)
    for r in range(n_req):
        q_off[r + 1] = q_off[r] + w.requests[r].n_q
    ctx = [w.ctx_len(r) for r in range(n_req)]
    tot_q = int(q_off[-1])
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, n_req, tot_q, max(ctx) + 300))
    reqs = [(rq.packet_ids, 0) for rq in w.requests]
    outs, tails = [dict() for _ in range(n_req)], [dict() for _ in range(n_req)]
    for layer in layers:
        parts = []
        for r in range(n_req):
            q, kn, vn = w.query(r, layer, "cuda")
            if prerotate_with is not None:
                q, kn = prerotate_with(r, layer, q, kn, ctx[r])
            parts.append((q, kn, vn))
        q, kn, vn = (torch.cat([p[i] for p in parts]).contiguous() for i in range(3))
        out = torch.full_like(q, float("nan"))
        k_tail = torch.full_like(kn, float("nan"))
        kvp.kvp_prefill_packets(store, reqs, layer, q, kn, vn, q_off, k_tail, ws, out, flags)
        torch.cuda.synchronize()
        for r in range(n_req):
            outs[r][layer] = out[q_off[r]:q_off[r + 1]].float().cpu().numpy().astype(np.float64)
            tails[r][layer] = W.to_numpy(k_tail[q_off[r]:q_off[r + 1]])
    return outs, tails


def _check_packets(w, layers, outs, tails, ref):
    worst = 0.0
    for r, rq in enumerate(w.requests):
        if rq.n_q == 0:
            continue
        ctx = ref["ctx"][r]
        for layer in layers:
            worst = max(worst, check_output(outs[r][layer], ref["out"][r][layer], "bf16", (w.name, r, layer)))
            # rotated K_new: the rows the cache path would have appended, bit for bit
            want = ref["k"][r][layer][:, ctx:ctx + rq.n_q].transpose(1, 0, 2)     # [n_q][Hkv][d]
            assert np.array_equal(tails[r][layer], want), (w.name, "k_tail", r, layer)
    return worst


@pytest.mark.parametrize("mk", [
    lambda: W.llama_k5(n_layers=2, n_packets=16),
    lambda: W.qwen_k20(n_layers=1, n_packets=40),
    lambda: W.llama_8k(n_layers=1, n_packets=16),
])
def test_prefill_packets_matches_oracle(gpu_device, mk):
    """Attention read in place from the store (no cache) gives the assembled path's result."""
    w = mk()
    layers = list(range(w.n_layers))
    outs, tails = _run_packets(w, layers)
    err = _check_packets(w, layers, outs, tails, oracle_workload(w))
    print(w.name, "in-place max abs err", err)


def test_prefill_packets_batch_ragged(gpu_device):
    w = W.llama_long_b8(n_layers=1, n_packets=6, batch=4, k=4, n_q=150)
    w.packet_lens[:] = [70, 1, 64, 129, 300, 63]
    w.requests[1].packet_ids = [2, 2, 5, 2]
    w.requests[2].n_q = 0
    w.requests[3].packet_ids = []            # no documents: causal self-attention of the query
    w.requests[3].n_q = 77
    outs, tails = _run_packets(w, [0])
    _check_packets(w, [0], outs, tails, oracle_workload(w))


def test_prefill_packets_split_invariance(gpu_device):
    w = W.llama_k5(n_layers=1, n_packets=8)
    ref = oracle_workload(w)
    for target in ("1", "64", "4000"):
        os.environ["KVP_ATTN_TARGET_ITEMS"] = target
        try:
            outs, tails = _run_packets(w, [0])
        finally:
            del os.environ["KVP_ATTN_TARGET_ITEMS"]
        _check_packets(w, [0], outs, tails, ref)


def test_a_prompt_prefix_is_a_first_packet_for_the_in_place_path(gpu_device):
    """Sec. 6.2 has a task prompt ahead of the documents.  The cache path takes it as rows the
    caller has written below base_pos; the in-place path has no cache to find such rows in and
    takes base_pos = 0 only: there the prompt's K/V is stored as a packet of its own (no adapter
    rows) and named first.  Both are the same composition -- the first packet sits at Delta = 0,
    which rotates nothing -- so one oracle run (the prompt as first packet) checks both."""
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=2, n_packets=8)
    w.packet_lens[w.requests[0].packet_ids[0]] = 37           # the "prompt": a short first packet
    rq = w.requests[0]
    prompt, docs, P = rq.packet_ids[0], rq.packet_ids[1:], 37
    ref = oracle_workload(w)
    layers = [0, 1]
    # in place: the prompt is one more packet
    outs, tails = _run_packets(w, layers)
    _check_packets(w, layers, outs, tails, ref)
    # cache path: the caller lays the prompt's rows into the cache and passes base_pos
    store = build_store(w, kvp)
    cache = make_cache(w, kvp, store)
    pk, pv = w.packet_kv(prompt, device="cuda")
    cache.k[0, :, :, :P], cache.v[0, :, :, :P] = pk, pv
    kvp.kvp_assemble(store, [(docs, P)], cache)
    ctx = int(cache.ctx_len[0])
    assert ctx == w.ctx_len(0)
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, rq.n_q, ctx + rq.n_q))
    with pytest.raises(kvp.KvpError) as e:                      # the in-place path says so when asked for base_pos
        kvp.kvp_prefill_packets(store, [(docs, P)], 0, *w.query(0, 0, "cuda"), [0, rq.n_q],
                                torch.empty(rq.n_q, 8, 128, dtype=torch.bfloat16, device="cuda"), ws,
                                torch.empty(rq.n_q, 32, 128, dtype=torch.bfloat16, device="cuda"))
    assert e.value.code == kvp.KVP_E_INVAL and "base_pos" in str(e.value)
    for layer in layers:
        q, kn, vn = w.query(0, layer, "cuda")
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, layer, q, kn, vn, [0, rq.n_q], ws, out)
        torch.cuda.synchronize()
        check_output(out.float().cpu().numpy().astype(np.float64), ref["out"][0][layer], w.dtype, ("prefix", layer))
        kg, vg = (W.to_numpy(x) for x in cache.logical(0, layer, ctx + rq.n_q))
        assert np.array_equal(kg, ref["k"][0][layer]) and np.array_equal(vg, ref["v"][0][layer])


def _compare_sampled(w, got, ref, sample, layers):
    for r in sample:
        rows = ref["ctx"][r] + w.requests[r].n_q
        for layer in layers:
            assert np.array_equal(got["k"][r][layer][:, :rows], ref["k"][r][layer][:, :rows]), (w.name, "K", r, layer)
            assert np.array_equal(got["v"][r][layer][:, :rows], ref["v"][r][layer][:, :rows]), (w.name, "V", r, layer)
            check_output(got["out"][r][layer], ref["out"][r][layer], w.dtype, (w.name, r, layer))


def test_full_size_llama_8k_sampled(gpu_device):
    """The benchmark's workload at full depth: assembly bit-exact on every layer (one launch
    over 32 layers), attention checked on two layers."""
    w = W.llama_8k()
    layers = [5, 31]
    got = run_workload(w, layers=layers)
    ref = oracle_workload(w, layers=layers)
    ctx = ref["ctx"][0]
    for layer in range(w.n_layers):
        rows = ctx + (w.requests[0].n_q if layer in layers else 0)
        assert np.array_equal(got["k"][0][layer][:, :rows], ref["k"][0][layer][:, :rows]), layer
        assert np.array_equal(got["v"][0][layer][:, :rows], ref["v"][0][layer][:, :rows]), layer
    for layer in layers:
        check_output(got["out"][0][layer], ref["out"][0][layer], w.dtype, (w.name, layer))


def test_full_size_long_context_batch_sampled(gpu_device):
    """Config 4 (batch 8, 32 packets of 528 rows, 128 query rows) on one layer: the oracle
    checks two of the eight requests."""
    w = W.llama_long_b8(n_layers=1)
    sample = [0, 5]
    got = run_workload(w)
    _compare_sampled(w, got, oracle_workload(w, requests=sample), sample, [0])


@pytest.mark.parametrize("n_q", [32, 1])
def test_full_size_long_context_few_query_rows_sampled(gpu_device, n_q):
    """The long-context batch with 32 query rows, and one decode step over it: HBM-bound launches
    that stream many tiles per compute unit, which the planner gives to 8-wave workgroups whose
    two wave groups take alternate tiles (merged through LDS) with one work item per CU."""
    import paper_2604_13226_amd as kvp
    w = W.llama_long_b8(n_layers=1, n_q=n_q)
    sample = [1, 6]
    got = run_workload(w)
    plan = kvp.kvp_debug_last_plan(got["store"], 1)
    assert plan[1] == 128 and 200 <= plan[3] <= 264                        # 128-row blocks, about one item per CU
    _compare_sampled(w, got, oracle_workload(w, requests=sample), sample, [0])


@pytest.mark.parametrize("paged", [False, True])
def test_two_wave_groups_on_alternate_tiles(gpu_device, paged):
    """The 8-wave shape of 128-row blocks forced on small ragged requests: odd and even tile
    counts, a single tile, items split over KV and unsplit, query rows inside the last tile."""
    w = W.llama_long_b8(n_layers=2, n_packets=6, batch=4, k=3, n_q=30)
    w.packet_lens[:] = [700, 130, 64, 529, 300, 63]
    w.requests[1].packet_ids = [2]                 # one tile of context
    w.requests[1].n_q = 5
    w.requests[2].packet_ids = []                  # no context at all
    w.requests[3].n_q = 1
    w.paged = paged
    ref = oracle_workload(w)
    for target in (None, "2000"):
        os.environ["KVP_ATTN_SPLIT_IN_WG"] = "1"
        if target:
            os.environ["KVP_ATTN_TARGET_ITEMS"] = target
        try:
            got = run_workload(w)
        finally:
            os.environ.pop("KVP_ATTN_SPLIT_IN_WG", None)
            os.environ.pop("KVP_ATTN_TARGET_ITEMS", None)
        compare(w, got, ref)


def test_paged_context_longer_than_one_items_block_ids(gpu_device):
    """A paged context of 34 K rows with one work item asked for: the item limit of 2047 block
    ids forces two kv ranges, merged by the combine kernel."""
    w = W.llama_long_b8(n_layers=1, n_packets=4, batch=1, k=4, n_q=6)
    w.n_q_heads, w.n_kv_heads = 8, 2
    w.packet_lens[:] = [16000, 9000, 8990, 40]
    w.requests[0].packet_ids = [0, 1, 2, 3]
    w.paged = True
    os.environ["KVP_ATTN_TARGET_ITEMS"] = "1"
    try:
        got = run_workload(w)
    finally:
        os.environ.pop("KVP_ATTN_TARGET_ITEMS", None)
    import paper_2604_13226_amd as kvp
    plan = kvp.kvp_debug_last_plan(got["store"], 1)
    assert plan[3] == 2 * 2                                   # two kv heads x two forced ranges
    compare(w, got, oracle_workload(w))


def test_context_of_128k_rows(gpu_device):
    """The longest context the paper's models take (131 072 positions): 64 packets of 2048 rows,
    32 query tokens, one layer.  Rotation angles at the far end, 2048 tiles, 32-way split."""
    w = W.llama_8k(n_layers=1, n_packets=16)
    w.packet_lens[:] = 2048
    w.requests[0].packet_ids = [int(x) for x in np.random.default_rng(5).integers(0, 8, size=64)]
    assert w.ctx_len(0) == 131072
    compare(w, run_workload(w), oracle_workload(w))


def test_full_size_serving_mix_sampled(gpu_device):
    """Config 5 (64 requests, paged cache, block 16, Zipf retrieval) on one layer: the oracle
    checks four of the 64 requests, among them the longest and the shortest context."""
    w = W.serving_mix(n_layers=1)
    ctx = [w.ctx_len(r) for r in range(len(w.requests))]
    sample = sorted({int(np.argmax(ctx)), int(np.argmin(ctx)), 7, 41})
    got = run_workload(w)
    _compare_sampled(w, got, oracle_workload(w, requests=sample), sample, [0])


def test_host_pinned_arena(gpu_device):
    """The packets wait in pinned host memory (the paper's tier, Sec. 5.1) and are read over
    PCIe in place: assembly stays bit-exact, both attention paths match the oracle."""
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=2, n_packets=8)
    ref = oracle_workload(w)
    store = build_store(w, kvp, arena="host")
    assert kvp.kvp_store_arena_on_host(store) == 1
    assert store.arena.is_pinned() and not store.arena.is_cuda
    got = run_workload(w, store=store)
    compare(w, got, ref)
    outs, tails = _run_packets(w, [0, 1], arena="host")
    _check_packets(w, [0, 1], outs, tails, ref)
    dev_store = build_store(w, kvp)
    assert kvp.kvp_store_arena_on_host(dev_store) == 0


def test_host_store_assembled_layer_group_by_layer_group_under_the_prefill(gpu_device):
    """The paper's own tier as a pipeline (Sec. 5.1: packets wait in CPU memory and are loaded on
    retrieval; Sec. 5.2: that copy is inside the time to first token): the store is pinned host
    memory, kvp_assemble brings one group of layers at a time over PCIe on a side stream while
    the main stream attends to the group before it.  ready[g] orders a group's prefill behind its
    assembly, free[g] orders the NEXT step's assembly of that group behind this step's prefill.
    Two steps back to back with different retrieval orders, so that an assembly that overtakes
    the previous step's prefill, or a prefill that overtakes its own assembly, changes an output."""
    import paper_2604_13226_amd as kvp
    wa = W.llama_k5(n_layers=4, n_packets=8)
    wb = W.llama_k5(n_layers=4, n_packets=8)
    wb.requests = [W.Request(list(wa.requests[0].packet_ids[::-1]), wa.requests[0].n_q)]
    refs = [oracle_workload(wa), oracle_workload(wb)]
    store = build_store(wa, kvp, arena="host")
    assert kvp.kvp_store_arena_on_host(store) == 1
    cache = make_cache(wa, kvp, store)
    n_q, L, G = wa.requests[0].n_q, wa.n_layers, 2
    ctx = wa.ctx_len(0)
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, n_q, ctx + n_q))
    qkv = [[w.query(0, layer, "cuda") for layer in range(L)] for w in (wa, wb)]
    outs = [[torch.full_like(qkv[0][0][0], float("nan")) for _ in range(L)] for _ in range(2)]
    side, main = torch.cuda.Stream(), torch.cuda.current_stream()
    ready = [torch.cuda.Event() for _ in range(L // G)]
    free = [torch.cuda.Event() for _ in range(L // G)]
    for e in free:
        e.record(main)
    torch.cuda.synchronize()
    for step, w in enumerate((wa, wb)):
        reqs = [(w.requests[0].packet_ids, 0)]
        for gi in range(L // G):                       # every group's assembly is queued on the side stream at once
            side.wait_event(free[gi])
            kvp.kvp_assemble(store, reqs, cache, gi * G, (gi + 1) * G, stream=side)
            ready[gi].record(side)
        for layer in range(L):
            if layer % G == 0:
                main.wait_event(ready[layer // G])
            q, kn, vn = qkv[step][layer]
            kvp.kvp_query_prefill(store, cache, layer, q, kn, vn, [0, n_q], ws, outs[step][layer], stream=main)
            if layer % G == G - 1:
                free[layer // G].record(main)
        assert int(cache.ctx_len[0]) == ctx
    torch.cuda.synchronize()
    for step, w in enumerate((wa, wb)):
        for layer in range(L):
            o = outs[step][layer].float().cpu().numpy().astype(np.float64)
            check_output(o, refs[step]["out"][0][layer], w.dtype, ("pipelined", step, layer))
    # the cache now holds the second step's rows, query rows included, bit for bit
    for layer in range(L):
        kg, vg = (W.to_numpy(x) for x in cache.logical(0, layer, ctx + n_q))
        assert np.array_equal(kg, refs[1]["k"][0][layer]), ("K", layer)
        assert np.array_equal(vg, refs[1]["v"][0][layer]), ("V", layer)
    # the two orders really differ (else the test would not notice a reordering)
    assert not np.array_equal(refs[0]["k"][0][0], refs[1]["k"][0][0])
    a, b = refs[0]["out"][0][0], refs[1]["out"][0][0]
    assert np.sqrt(np.mean((a - b) ** 2)) > 20 * REL_RMS_TOL["bf16"] * np.sqrt(np.mean(b * b))   # far beyond check_output's relative bar


def _compressed_case(w, seed, keep_prob, compressed_ids):
    """Per packet and layer the sorted rows a pruning pass kept (None: the packet stays whole)."""
    rng = np.random.default_rng(seed)
    keeps = {}
    for p in sorted({p for rq in w.requests for p in rq.packet_ids}):
        L = int(w.packet_lens[p])
        if p not in compressed_ids:
            keeps[p] = None
            continue
        keeps[p] = [np.flatnonzero(rng.random(L) < keep_prob) for _ in range(w.n_layers)]
    return keeps


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_compressed_packets_match_oracle(gpu_device, dtype, paged):
    """Sec. 5.4: packets whose layers kept different row subsets are realigned by the Delta of
    their uncompressed spans and concatenated without gaps; assembly bit-exact per layer (rows
    and their count), attention within tolerance with the query at the position after the spans."""
    import paper_2604_13226_amd as kvp
    import oracle
    if dtype == "bf16":
        w = W.llama_k5(n_layers=3, n_packets=6)
        w.packet_lens[:] = [300, 65, 128, 1, 517, 64]
        w.requests[0].packet_ids = [4, 1, 0, 3, 2]
        w.requests.append(W.Request(packet_ids=[5, 0], n_q=7, base_pos=0))     # a whole packet, then a compressed one
        w.requests.append(W.Request(packet_ids=[1], n_q=33, base_pos=3))
        comp = {0, 2, 3, 4}
    else:
        w = W.random_small(77, dtype="f32", d=64, n_q_heads=4, n_kv_heads=2, n_layers=2, n_packets=4, k=3, n_q=5, max_len=90)
        comp = {w.requests[0].packet_ids[0], w.requests[0].packet_ids[-1]}
        w.requests.append(W.Request(packet_ids=list(w.requests[0].packet_ids[::-1]), n_q=6, base_pos=5))
    w.paged = paged
    w.block_size = 16
    keeps = _compressed_case(w, 5, 0.55, comp)
    if dtype == "bf16":
        keeps[3] = [np.array([0]), np.array([], int), np.array([0])]          # a one-row packet, pruned away in layer 1
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    n_req, L = len(w.requests), w.n_layers
    spans = {p: int(w.packet_lens[p]) for p in keeps}

    # ---- library
    pk = {p: w.packet_kv(p, device="cuda") for p in keeps}
    arena = sum(kvp.packet_bytes(L, w.n_kv_heads, w.head_dim, w.dtype, spans[p]) for p in keeps) + 4096
    pos_q = [rq.base_pos + sum(spans[p] for p in rq.packet_ids) for rq in w.requests]
    store = kvp.kvp_store_create(L, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, w.rope_base,
                                 max(pos_q) + 64, arena, w.n_header, w.n_trailer, device=0)
    for p, keep in keeps.items():
        k, v = pk[p]
        if keep is None:
            kvp.kvp_store_put(store, p, k, v)
        else:
            idx = [torch.as_tensor(kk, device="cuda") for kk in keep]
            kvp.kvp_store_put_compressed(store, p, spans[p], [k[l][:, idx[l]].contiguous() for l in range(L)],
                                         [v[l][:, idx[l]].contiguous() for l in range(L)])
    rows_max = max(pos_q) + max(rq.n_q for rq in w.requests)
    if paged:
        bs = 16
        nblk = [(pos_q[r] + w.requests[r].n_q + bs - 1) // bs for r in range(n_req)]
        total = sum(nblk) + 2
        perm = np.random.default_rng(9).permutation(total)
        table = np.zeros((n_req, max(nblk)), np.int32)
        at = 0
        for r in range(n_req):
            table[r, :nblk[r]] = perm[at:at + nblk[r]]
            at += nblk[r]
        cache = kvp.Cache.paged(store, n_req, total, table, bs)
    else:
        cache = kvp.Cache.contiguous(store, n_req, rows_max + 3)
    cache.with_ctx_rows(L)
    kvp.kvp_assemble(store, [(rq.packet_ids, rq.base_pos) for rq in w.requests], cache)
    assert [int(x) for x in cache.ctx_len[:n_req]] == pos_q
    # the caller's own rows below base_pos (a prompt prefix): seeded values, laid into the cache
    # by the test as a caller would, keys as they are (already at positions 0 .. base_pos - 1)
    prefix = {}
    for r, rq in enumerate(w.requests):
        for layer in range(L):
            if rq.base_pos:
                pk_, pv_ = (W.normal_tensor((w.n_kv_heads, rq.base_pos, w.head_dim), 4321, 10 + i, r * 64 + layer, w.kv_scale,
                                            w.torch_dtype, "cuda") for i in range(2))
                prefix[r, layer] = (W.to_numpy(pk_), W.to_numpy(pv_))
                for t in range(rq.base_pos):
                    if paged:
                        blk, slot = int(cache.block_table[r, t // 16]), t % 16
                        cache.k[layer, blk, :, slot], cache.v[layer, blk, :, slot] = pk_[:, t], pv_[:, t]
                    else:
                        cache.k[r, layer, :, t], cache.v[r, layer, :, t] = pk_[:, t], pv_[:, t]
    q_off = np.zeros(n_req + 1, np.int32)
    for r in range(n_req):
        q_off[r + 1] = q_off[r] + w.requests[r].n_q
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, n_req, int(q_off[-1]), rows_max))
    outs = {}
    for layer in range(L):
        parts = [w.query(r, layer, "cuda") for r in range(n_req)]
        q, kn, vn = (torch.cat([p_[i] for p_ in parts]).contiguous() for i in range(3))
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, layer, q, kn, vn, q_off, ws, out)
        torch.cuda.synchronize()
        outs[layer] = out.float().cpu().numpy().astype(np.float64)

    # ---- oracle, layer by layer
    for r, rq in enumerate(w.requests):
        for layer in range(L):
            ks, vs = [], []
            for p in rq.packet_ids:
                k, v = (W.to_numpy(x) for x in w.packet_kv(p))
                sel = np.arange(spans[p]) if keeps[p] is None else keeps[p][layer]
                ks.append(np.ascontiguousarray(k[layer][:, sel]))
                vs.append(np.ascontiguousarray(v[layer][:, sel]))
            n_rows = rq.base_pos + sum(k.shape[1] for k in ks)
            Ko, Vo, rows, pos_end = oracle.assemble_layer_spans(w.dtype, ks, vs, [spans[p] for p in rq.packet_ids], f,
                                                                rq.base_pos, t_cap=n_rows - rq.base_pos + rq.n_q)
            assert pos_end == pos_q[r]
            assert int(cache.ctx_rows[r][layer]) == n_rows
            # the oracle's layer starts at the first packet row; the cache has base_pos caller rows before it
            kg, vg = cache.logical(r, layer, n_rows + rq.n_q)
            kg, vg = W.to_numpy(kg)[:, rq.base_pos:], W.to_numpy(vg)[:, rq.base_pos:]
            assert np.array_equal(kg[:, :rows], Ko[:, :rows]), (r, layer, "K")
            assert np.array_equal(vg[:, :rows], Vo[:, :rows]), (r, layer, "V")
            qq, kn, vn = (W.to_numpy(x) for x in w.query(r, layer))
            if rq.base_pos:
                # the caller's rows take part in attention: the oracle's layer gets them in front of
                # the packets' rows; rows and positions are now shifted by different amounts
                # (rows: base_pos + kept rows, positions: base_pos + spans)
                Kf = np.concatenate([prefix[r, layer][0], Ko], axis=1)
                Vf = np.concatenate([prefix[r, layer][1], Vo], axis=1)
                ref = oracle.query_prefill_at(w.dtype, qq, kn, vn, f, rq.base_pos + rows, pos_end, Kf, Vf)
                Ko, Vo = Kf[:, rq.base_pos:], Vf[:, rq.base_pos:]
            else:
                ref = oracle.query_prefill_at(w.dtype, qq, kn, vn, f, rows, pos_end, Ko, Vo)
            assert np.array_equal(kg[:, rows:rows + rq.n_q], Ko[:, rows:rows + rq.n_q]), (r, layer, "K_new")
            assert np.array_equal(vg[:, rows:rows + rq.n_q], Vo[:, rows:rows + rq.n_q]), (r, layer, "V_new")
            check_output(outs[layer][q_off[r]:q_off[r + 1]], ref, w.dtype, ("compressed", r, layer))


def test_pruned_headline_workload(gpu_device):
    """The benchmark's pruned workload (Sec. 5.4, 10-50 % of every packet's rows removed, another
    subset in every layer) at its full context, six layers of it (96 segments: the gather plan is
    uploaded and searched, not carried in the kernel arguments): one assembly launch over all
    layers, rows of every layer bit-exact, attention within tolerance."""
    import paper_2604_13226_amd as kvp
    import oracle
    w = W.llama_8k_pruned(n_layers=6, n_packets=16)
    rq = w.requests[0]
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    store = build_store(w, kvp)
    cache = make_cache(w, kvp, store)
    kvp.kvp_assemble(store, [(rq.packet_ids, 0)], cache)
    assert int(cache.ctx_len[0]) == w.ctx_len(0)
    n_q = rq.n_q
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, n_q, w.ctx_len(0) + n_q))
    spans = [int(w.packet_lens[p]) for p in rq.packet_ids]
    kv = [tuple(W.to_numpy(x) for x in w.packet_kv(p)) for p in rq.packet_ids]
    first_pass = []
    for layer in range(w.n_layers):
        q, kn, vn = w.query(0, layer, "cuda")
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, layer, q, kn, vn, [0, n_q], ws, out)
        torch.cuda.synchronize()
        keep = [w.kept_rows(p, layer) for p in rq.packet_ids]
        ks = [np.ascontiguousarray(k[layer][:, s]) for (k, _), s in zip(kv, keep)]
        vs = [np.ascontiguousarray(v[layer][:, s]) for (_, v), s in zip(kv, keep)]
        Ko, Vo, rows, pos_end = oracle.assemble_layer_spans(w.dtype, ks, vs, spans, f, 0, t_cap=w.layer_rows(0, layer) + n_q)
        assert rows == w.layer_rows(0, layer) == int(cache.ctx_rows[0][layer]) and pos_end == w.ctx_len(0)
        ref = oracle.query_prefill_at(w.dtype, *(W.to_numpy(x) for x in (q, kn, vn)), f, rows, pos_end, Ko, Vo)
        kg, vg = (W.to_numpy(x) for x in cache.logical(0, layer, rows + n_q))
        assert np.array_equal(kg, Ko[:, :rows + n_q]), (layer, "K")
        assert np.array_equal(vg, Vo[:, :rows + n_q]), (layer, "V")
        check_output(out.float().cpu().numpy().astype(np.float64), ref, w.dtype, ("pruned 8k", layer))
        first_pass.append(out)
    # every layer has its own plan; a second pass finds them again and gives the same bits
    for layer in range(w.n_layers):
        q, kn, vn = w.query(0, layer, "cuda")
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, layer, q, kn, vn, [0, n_q], ws, out)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), first_pass[layer].view(torch.int16)), layer


def _check_pruned_workload(w, tag):
    """A workload whose packets are all pruned (w.prune), any number of requests, base_pos 0:
    one assembly over all layers, then every layer's prefill, against the oracle layer by layer."""
    import paper_2604_13226_amd as kvp
    import oracle
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    n_req, L = len(w.requests), w.n_layers
    store = build_store(w, kvp)
    cache = make_cache(w, kvp, store)
    kvp.kvp_assemble(store, [(rq.packet_ids, 0) for rq in w.requests], cache)
    assert [int(x) for x in cache.ctx_len[:n_req]] == [w.ctx_len(r) for r in range(n_req)]
    q_off = np.zeros(n_req + 1, np.int32)
    for r in range(n_req):
        q_off[r + 1] = q_off[r] + w.requests[r].n_q
    rows_max = max(w.ctx_len(r) + w.requests[r].n_q for r in range(n_req))
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, n_req, int(q_off[-1]), rows_max))
    for layer in range(L):
        parts = [w.query(r, layer, "cuda") for r in range(n_req)]
        q, kn, vn = (torch.cat([p_[i] for p_ in parts]).contiguous() for i in range(3))
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, layer, q, kn, vn, q_off, ws, out)
        torch.cuda.synchronize()
        out = out.float().cpu().numpy().astype(np.float64)
        for r, rq in enumerate(w.requests):
            kv = [tuple(W.to_numpy(x) for x in w.packet_kv(p)) for p in rq.packet_ids]
            keep = [w.kept_rows(p, layer) for p in rq.packet_ids]
            ks = [np.ascontiguousarray(k[layer][:, s_]) for (k, _), s_ in zip(kv, keep)]
            vs = [np.ascontiguousarray(v[layer][:, s_]) for (_, v), s_ in zip(kv, keep)]
            spans = [int(w.packet_lens[p]) for p in rq.packet_ids]
            rows_l = w.layer_rows(r, layer)
            if ks:
                Ko, Vo, rows, pos_end = oracle.assemble_layer_spans(w.dtype, ks, vs, spans, f, 0, t_cap=rows_l + rq.n_q)
            else:                      # no packets: an empty layer for the query rows to go into
                Ko = np.zeros((w.n_kv_heads, rq.n_q, w.head_dim), np.float32 if w.dtype == "f32" else np.uint16)
                Vo, rows, pos_end = Ko.copy(), 0, 0
            assert rows == rows_l == int(cache.ctx_rows[r][layer]) and pos_end == w.ctx_len(r)
            if rq.n_q == 0 and not ks:
                continue
            ref = oracle.query_prefill_at(w.dtype, *(W.to_numpy(x) for x in parts[r]), f, rows, pos_end, Ko, Vo)
            kg, vg = (W.to_numpy(x) for x in cache.logical(r, layer, rows + rq.n_q))
            assert np.array_equal(kg, Ko[:, :rows + rq.n_q]), (tag, r, layer, "K")
            assert np.array_equal(vg, Vo[:, :rows + rq.n_q]), (tag, r, layer, "V")
            if rq.n_q:
                check_output(out[q_off[r]:q_off[r + 1]], ref, w.dtype, (tag, r, layer))


@pytest.mark.parametrize("seed", range(500, 516))
def test_random_geometries_pruned(gpu_device, seed):
    """Seeded random batches whose packets are all pruned, a different subset in every layer."""
    w = _random_geometry(seed)
    rng = np.random.default_rng(seed + 1)
    for rq in w.requests:
        rq.base_pos = 0
    w.shared_header = False
    w.n_layers = int(rng.integers(1, 4))
    lo = float(rng.uniform(0.0, 0.6))
    w.prune = (lo, min(1.0, lo + float(rng.uniform(0.0, 0.5))))
    _check_pruned_workload(w, ("pruned", seed))


@pytest.mark.parametrize("seed", range(600, 612))
def test_random_geometries_pruned_in_place(gpu_device, seed):
    """Pruned packets read in place (kvp_prefill_packets): every layer tiles its own kept rows;
    the oracle composes that layer from the kept rows and attends with the query at the position
    after the spans."""
    import oracle
    rng = np.random.default_rng(seed)
    n_req, n_packets = int(rng.integers(1, 4)), int(rng.integers(2, 6))
    g, n_kv = int(rng.choice([1, 4])), int(rng.choice([1, 2]))
    w = W.random_small(seed, dtype="bf16", d=128, n_q_heads=n_kv * g, n_kv_heads=n_kv, n_layers=int(rng.integers(1, 4)),
                       n_packets=n_packets, k=1, n_q=1, max_len=int(rng.choice([9, 70, 300])), n_req=n_req)
    for rq in w.requests:
        rq.packet_ids = [int(x) for x in rng.integers(0, n_packets, size=int(rng.integers(0, 5)))]
        rq.n_q = int(rng.integers(0, 100))
    if all(rq.n_q == 0 for rq in w.requests):
        w.requests[0].n_q = 3
    lo = float(rng.uniform(0.0, 0.6))
    w.prune = (lo, min(1.0, lo + float(rng.uniform(0.0, 0.5))))
    layers = list(range(w.n_layers))
    outs, tails = _run_packets(w, layers)
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    for r, rq in enumerate(w.requests):
        if rq.n_q == 0:
            continue
        kv = [tuple(W.to_numpy(x) for x in w.packet_kv(p)) for p in rq.packet_ids]
        spans = [int(w.packet_lens[p]) for p in rq.packet_ids]
        for layer in layers:
            keep = [w.kept_rows(p, layer) for p in rq.packet_ids]
            ks = [np.ascontiguousarray(k[layer][:, s_]) for (k, _), s_ in zip(kv, keep)]
            vs = [np.ascontiguousarray(v[layer][:, s_]) for (_, v), s_ in zip(kv, keep)]
            if ks:
                Ko, Vo, rows, pos_end = oracle.assemble_layer_spans(w.dtype, ks, vs, spans, f, 0, t_cap=w.layer_rows(r, layer) + rq.n_q)
            else:
                Ko = np.zeros((w.n_kv_heads, rq.n_q, w.head_dim), np.uint16)
                Vo, rows, pos_end = Ko.copy(), 0, 0
            ref = oracle.query_prefill_at(w.dtype, *(W.to_numpy(x) for x in w.query(r, layer)), f, rows, pos_end, Ko, Vo)
            check_output(outs[r][layer], ref, w.dtype, ("pruned in place", seed, r, layer))
            assert np.array_equal(tails[r][layer], Ko[:, rows:rows + rq.n_q].transpose(1, 0, 2)), (seed, "k_tail", r, layer)


@pytest.mark.parametrize("seed", range(400, 416))
def test_random_geometries_in_place(gpu_device, seed):
    """Seeded random bf16 batches through kvp_prefill_packets (attention in place, no cache)."""
    rng = np.random.default_rng(seed)
    n_req, n_packets = int(rng.integers(1, 5)), int(rng.integers(2, 7))
    g = int(rng.choice([1, 4, 7]))
    n_kv = int(rng.choice([1, 2, 4]))
    w = W.random_small(seed, dtype="bf16", d=128, n_q_heads=n_kv * g, n_kv_heads=n_kv, n_layers=int(rng.integers(1, 3)),
                       n_packets=n_packets, k=1, n_q=1, max_len=int(rng.choice([9, 70, 300, 700])), n_req=n_req)
    for rq in w.requests:
        rq.packet_ids = [int(x) for x in rng.integers(0, n_packets, size=int(rng.integers(0, 6)))]
        rq.n_q = int(rng.integers(0, 150))
    if all(rq.n_q == 0 for rq in w.requests):
        w.requests[0].n_q = 3
    if rng.random() < 0.4:
        w.n_header, w.shared_header = int(rng.choice([1, 4, 8])), True
    w.name = "in place %d" % seed
    layers = list(range(w.n_layers))
    env = {}
    if seed >= 408:  # the second half with the planner's choices overridden at random
        env["KVP_ATTN_TARGET_ITEMS"] = str(int(rng.choice([1, 7, 64, 300, 4000])))
        if rng.random() < 0.5:
            env["KVP_ATTN_BM"] = str(int(rng.choice([128, 256])))
        if rng.random() < 0.5:
            env["KVP_ATTN_SPLIT_IN_WG"] = str(int(rng.integers(0, 2)))
        if rng.random() < 0.3:
            env["KVP_ATTN_MIXED"] = "0"
        if rng.random() < 0.4:
            env["KVP_ATTN_NT_LOADS"] = str(int(rng.integers(0, 2)))
    os.environ.update(env)
    try:
        outs, tails = _run_packets(w, layers)
    finally:
        for k in env:
            os.environ.pop(k, None)
    try:
        _check_packets(w, layers, outs, tails, oracle_workload(w))
    except AssertionError as e:
        raise AssertionError("with %s: %s" % (env, e))


@pytest.mark.parametrize("case", ["bf16", "bf16 paged", "f32", "mixed with compressed"])
def test_shared_header_store_matches_whole_packets(gpu_device, case):
    """Sec. 4.1: the header is global, so its rows are the same in every packet and the store may
    hold them once (kvp_store_put_header / kvp_store_put_body).  The oracle composes the whole
    packets; the library reads the header rows from the shared copy: cache rows bit-exact,
    attention within tolerance, on both the assembled and the in-place path."""
    import paper_2604_13226_amd as kvp
    if case == "f32":
        w = W.random_small(91, dtype="f32", d=64, n_q_heads=4, n_kv_heads=2, n_layers=2, n_packets=5, k=4, n_q=6,
                           max_len=50, n_req=2, base_pos=3)
        w.n_header, w.n_trailer = 3, 2
        w.packet_lens[0] = 2                        # shorter than the header: stored whole
    else:
        w = W.llama_long_b8(n_layers=2, n_packets=6, batch=3, k=4, n_q=40)
        w.packet_lens[:] = [70, 9, 64, 129, 300, 8]   # 9: one body row; 8: header only, stored whole
        w.requests[1].packet_ids = [2, 2, 5, 1]
        w.requests[2].n_q = 3
        w.paged = case == "bf16 paged"
    w.shared_header = True
    ref = oracle_workload(w)
    if case != "mixed with compressed":
        compare(w, run_workload(w), ref)
        if w.dtype == "bf16" and not w.paged:
            layers = list(range(w.n_layers))
            outs, tails = _run_packets(w, layers)
            _check_packets(w, layers, outs, tails, ref)
        return
    # a compressed packet in the request sends the call down the layer-by-layer route, where the
    # header-less packets get a header segment per layer; keeping every row of the compressed
    # packet makes the whole-packet oracle the reference
    store = build_store(w, kvp, packets=[0, 1, 2, 3, 5], extra_bytes=1 << 24)
    k4, v4 = w.packet_kv(4, "cuda")
    kvp.kvp_store_put_compressed(store, 4, 300, [k4[l].contiguous() for l in range(w.n_layers)],
                                 [v4[l].contiguous() for l in range(w.n_layers)])
    w.requests[0].packet_ids = [3, 4, 0, 1]
    ref = oracle_workload(w)
    cache = make_cache(w, kvp, store).with_ctx_rows(w.n_layers)
    kvp.kvp_assemble(store, [(rq.packet_ids, rq.base_pos) for rq in w.requests], cache)
    for r in range(len(w.requests)):
        for layer in range(w.n_layers):
            ctx = w.ctx_len(r)
            assert int(cache.ctx_rows[r][layer]) == ctx == int(cache.ctx_len[r])
            k, v = cache.logical(r, layer, ctx)
            assert np.array_equal(W.to_numpy(k), ref["k"][r][layer][:, :ctx]), (r, layer, "K")
            assert np.array_equal(W.to_numpy(v), ref["v"][r][layer][:, :ctx]), (r, layer, "V")


def test_repeated_calls_reuse_the_plan_and_give_the_same_bits(gpu_device):
    """The same geometry layer after layer reuses the uploaded plan: six calls in a row match the
    oracle and each other bit for bit (same items, same merge order)."""
    import paper_2604_13226_amd as kvp
    w = W.llama_8k(n_layers=1, n_packets=16)
    ref = oracle_workload(w)
    store = build_store(w, kvp)
    cache = make_cache(w, kvp, store)
    kvp.kvp_assemble(store, [(rq.packet_ids, rq.base_pos) for rq in w.requests], cache)
    q, kn, vn = w.query(0, 0, "cuda")
    n_q = w.requests[0].n_q
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, n_q, w.ctx_len(0) + n_q))
    outs = []
    for rep in range(6):
        out = torch.full_like(q, float("nan"))
        kvp.kvp_query_prefill(store, cache, 0, q, kn, vn, [0, n_q], ws, out)
        torch.cuda.synchronize()
        o = out.float().cpu().numpy().astype(np.float64)
        check_output(o, ref["out"][0][0], w.dtype, ("repeat", rep))
        outs.append(o)
    assert kvp.kvp_debug_last_plan(store, 1)[3] > 8          # the call was split
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])


def test_a_gather_plan_kept_on_the_device_serves_the_same_call_again_and_no_other(gpu_device):
    """A paged assembly uploads its plan (segments, tile map, block table); the same call again
    launches from the kept copy, a call with another block table or other requests does not.
    Every pass is checked bit for bit against the oracle after the caches were overwritten, on
    more calls than the library keeps plans for."""
    import paper_2604_13226_amd as kvp
    w = W.serving_mix(n_layers=1, n_packets=64, n_req=5)
    ref = oracle_workload(w)
    store = build_store(w, kvp)
    reqs = [(rq.packet_ids, rq.base_pos) for rq in w.requests]

    def check(cache, ref_, n_req):
        torch.cuda.synchronize()
        for r in range(n_req):
            k, v = cache.logical(r, 0, ref_["ctx"][r])
            assert np.array_equal(W.to_numpy(k), ref_["k"][r][0][:, :ref_["ctx"][r]]), r
            assert np.array_equal(W.to_numpy(v), ref_["v"][r][0][:, :ref_["ctx"][r]]), r

    c1 = make_cache(w, kvp, store, block_order="random")
    c2 = make_cache(w, kvp, store, block_order="sequential")     # same shapes, another block table
    for rep in range(3):
        for c in (c1, c2, c1):
            c.k.fill_(7.0), c.v.fill_(7.0)
            kvp.kvp_assemble(store, reqs, c)
            check(c, ref, len(reqs))
    # other requests on the same cache: fewer, in another order
    w2 = W.serving_mix(n_layers=1, n_packets=64, n_req=5)
    w2.requests = [w.requests[3], w.requests[0]]
    ref2 = oracle_workload(w2)
    c3 = make_cache(w2, kvp, store)
    for rep in range(12):                                        # more rewrites than there are kept plans
        c3.k.fill_(float(rep)), c3.v.fill_(float(rep))
        kvp.kvp_assemble(store, [(rq.packet_ids, rq.base_pos) for rq in w2.requests], c3)
        check(c3, ref2, 2)
        if rep % 4 == 0:
            c1.k.fill_(9.0), c1.v.fill_(9.0)
            kvp.kvp_assemble(store, reqs, c1)
            check(c1, ref, len(reqs))


def _with_lens(w, n):
    w.packet_lens[:] = n
    return w


@pytest.mark.parametrize("mk", [
    lambda: W.llama_k5(n_layers=1, n_packets=8),
    lambda: W.llama_8k(n_layers=1, n_packets=16),
    lambda: W.llama_8k(n_layers=1, n_packets=16, n_q=1),
    lambda: _with_lens(W.llama_8k(n_layers=1, n_packets=16), 526),      # 8416 + 32 rows = 22 x 384: the last kv range is a full one
])
def test_items_rebuilt_from_the_block_index_give_the_same_bits_as_items_read_from_memory(gpu_device, mk):
    """The workgroups of a regular one-request launch rebuild their work items from their index;
    with that switched off (KVP_ATTN_INLINE_ITEMS=0) the same items are read from memory.  Same
    items, same arithmetic: the outputs and the appended rows agree bit for bit, on both attention
    paths."""
    import paper_2604_13226_amd as kvp
    w = mk()
    res = {}
    for inline in ("1", "0"):
        os.environ["KVP_ATTN_INLINE_ITEMS"] = inline
        try:
            got = run_workload(w)
            n_inl = int(kvp.kvp_debug_last_plan(got["store"], 2)[0])
            assert (n_inl > 0) == (inline == "1")
            outs, tails = _run_packets(w, [0])
        finally:
            del os.environ["KVP_ATTN_INLINE_ITEMS"]
        res[inline] = (got["out"][0][0], got["k"][0][0], outs[0][0], tails[0][0])
    for a, b in zip(res["1"], res["0"]):
        assert np.array_equal(a, b)
    compare(w, got, oracle_workload(w))


def test_empty_batches_touch_nothing(gpu_device):
    """No requests, or requests without packets and without query rows: the calls succeed, launch
    nothing and leave the cache, the output and ctx_len of other requests alone."""
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=1, n_packets=8)
    store = build_store(w, kvp)
    cache = make_cache(w, kvp, store)
    cache.k.fill_(1.0)
    cache.v.fill_(1.0)
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, 8, 64))
    q, kn, vn = (x[:0].contiguous() for x in w.query(0, 0, "cuda"))
    out = torch.empty_like(q)
    none = np.array([0], np.int32)
    kvp.kvp_assemble(store, [], cache)
    kvp.kvp_query_prefill(store, cache, 0, q, kn, vn, none, ws, out)
    kvp.kvp_prefill_packets(store, [], 0, q, kn, vn, none, torch.empty_like(kn), ws, out)
    kvp.kvp_assemble(store, [([], 0)], cache)
    assert cache.ctx_len[0] == 0
    kvp.kvp_query_prefill(store, cache, 0, q, kn, vn, np.array([0, 0], np.int32), ws, out)
    kvp.kvp_prefill_packets(store, [([], 0)], 0, q, kn, vn, np.array([0, 0], np.int32), torch.empty_like(kn), ws, out)
    torch.cuda.synchronize()
    assert bool((cache.k == 1.0).all()) and bool((cache.v == 1.0).all())
    kvp.kvp_store_destroy(store)


@pytest.mark.filterwarnings("ignore:The CUDA Graph is empty")
@pytest.mark.parametrize("path", ["cache", "packets"])
def test_launches_replayed_from_a_graph(gpu_device, path):
    """A caller may capture the calls into a HIP graph (the per-layer launches of a short context
    are launch-bound) once the plan of the same geometry exists on that stream.  Every replay,
    with eager calls of other geometries and synchronisations in between (they would replace the
    captured plan if it were not kept), gives the bits of the eager run, which match the oracle."""
    import paper_2604_13226_amd as kvp
    w = W.llama_k5(n_layers=2, n_packets=8)
    rq = w.requests[0]
    rq.packet_ids, rq.n_q = rq.packet_ids[:3], 20
    ref = oracle_workload(w)
    store = build_store(w, kvp)
    cache = make_cache(w, kvp, store)
    reqs = [(rq.packet_ids, 0)]
    q_off = np.array([0, rq.n_q], np.int32)
    ws = kvp.alloc_workspace(kvp.kvp_prefill_workspace_bytes(store, 1, rq.n_q, w.ctx_len(0) + rq.n_q))
    qkv = [w.query(0, l, "cuda") for l in range(w.n_layers)]
    outs = [torch.empty_like(qkv[0][0]) for _ in range(w.n_layers)]
    k_tail = [torch.empty_like(qkv[0][1]) for _ in range(w.n_layers)]

    def calls():
        if path == "cache":
            kvp.kvp_assemble(store, reqs, cache)
        for l in range(w.n_layers):
            q, kn, vn = qkv[l]
            if path == "cache":
                kvp.kvp_query_prefill(store, cache, l, q, kn, vn, q_off, ws, outs[l])
            else:
                kvp.kvp_prefill_packets(store, reqs, l, q, kn, vn, q_off, k_tail[l], ws, outs[l])

    def other_geometries(n):  # eager calls with n other query lengths: each needs a plan of its own
        for i in range(n):
            nq = 1 + i
            q, kn, vn = (x[:nq].contiguous() for x in qkv[0])
            o = torch.empty_like(q)
            qo = np.array([0, nq], np.int32)
            if path == "cache":
                kvp.kvp_query_prefill(store, cache, 0, q, kn, vn, qo, ws, o)
            else:
                kvp.kvp_prefill_packets(store, reqs, 0, q, kn, vn, qo, torch.empty_like(kn), ws, o)

    def state():
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        if path == "cache":
            rows = w.ctx_len(0) + rq.n_q
            got += [x.clone() for l in range(w.n_layers) for x in cache.logical(0, l, rows)]
        else:
            got += [t.clone() for t in k_tail]
        return got

    def clobber():
        for t in outs + k_tail:
            t.fill_(float("nan"))
        if path == "cache":
            cache.k.zero_()
            cache.v.zero_()

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        # a geometry the stream has no plan for cannot be captured: the call says so, launches nothing
        empty = torch.cuda.CUDAGraph()
        with torch.cuda.graph(empty, stream=side):
            with pytest.raises(kvp.KvpError, match="capture"):
                if path == "cache":
                    kvp.kvp_query_prefill(store, cache, 0, *qkv[0], q_off, ws, outs[0])
                else:
                    kvp.kvp_prefill_packets(store, reqs, 0, *qkv[0], q_off, k_tail[0], ws, outs[0])
        calls()                               # eager: builds and keeps the plans
        eager = state()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            calls()
        for replay in range(3):
            other_geometries(12)              # more plans than the store keeps beside captured ones
            clobber()
            g.replay()
            now = state()
            for a, b in zip(eager, now):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), (path, replay)
        calls()                               # and eager calls still work next to the graph
        for a, b in zip(eager, state()):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    for l in range(w.n_layers):
        check_output(outs[l].float().cpu().numpy().astype(np.float64), ref["out"][0][l], w.dtype, (path, l))
    kvp.kvp_store_destroy(store)


def test_zz_report_worst_relative_rms(gpu_device):
    """Prints the largest relative rms error the tests above saw (run with -s to see it)."""
    print("worst relative rms error:", WORST_REL_RMS)
