"""CPU-only tests of the C-ABI library: it loads, exports what include/kvp.h declares, and
its host logic (directory, offsets Delta_j, gather tiles, split-KV plan, every error code)
is right.  A store created with KVP_DEVICE_NONE plans and validates but launches nothing."""
import os
import re

import numpy as np
import pytest

import paper_2604_13226_amd as kvp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def dry_store(**kw):
    a = dict(n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16", rope_base=5.0e5,
             max_positions=1 << 16, arena_bytes=1 << 30, n_header=8, n_trailer=8,
             device=kvp.KVP_DEVICE_NONE)
    a.update(kw)
    return kvp.kvp_store_create(**a)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "kvp.h")).read()
    declared = set(re.findall(r"\b(kvp_[a-z_]+)\s*\(", header))
    declared -= {"kvp_prefill_workspace_bytes()"}
    assert {"kvp_store_put", "kvp_assemble", "kvp_query_prefill"} <= declared
    lib = kvp.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert set(kvp.binding.EXPORTS) == declared
    assert kvp.kvp_version().startswith("kvp ")


@pytest.mark.parametrize("bad", [
    dict(head_dim=127), dict(head_dim=0), dict(head_dim=512), dict(n_q_heads=7),
    dict(n_layers=0), dict(dtype_code=5), dict(max_positions=0), dict(rope_base=-1.0),
    dict(n_header=-1),
])
def test_create_rejects_bad_config(bad):
    bad = dict(bad)
    code = bad.pop("dtype_code", None)
    if code is not None:
        kvp.binding._dtype_code  # noqa
        orig = kvp.binding._dtype_code
        kvp.binding._dtype_code = lambda _: code
        try:
            with pytest.raises(kvp.KvpError) as e:
                dry_store()
        finally:
            kvp.binding._dtype_code = orig
    else:
        with pytest.raises(kvp.KvpError) as e:
            dry_store(**bad)
    assert e.value.code == kvp.KVP_E_INVAL
    assert str(e.value)


def test_directory_and_arena_accounting():
    per100 = kvp.packet_bytes(2, 2, 128, "bf16", 100)
    raw100 = 2 * 2 * 2 * 100 * 128 * 2
    assert raw100 <= per100 <= raw100 * 1.05 and per100 % 256 == 0
    per200 = kvp.packet_bytes(2, 2, 128, "bf16", 200)
    s = dry_store(arena_bytes=per100 + per200)
    assert kvp.kvp_packet_bytes(s, 100) == per100
    assert kvp.kvp_packet_bytes(s, 1) == 2 * 2 * 2 * 128 * 2
    assert kvp.kvp_packet_bytes(s, 200) <= 2 * per100
    kvp.kvp_store_put(s, 7, None, None, n_tokens=100)
    assert kvp.kvp_store_packet_len(s, 7) == 100
    assert kvp.kvp_store_packet_len(s, 8) == kvp.KVP_E_NOTFOUND
    assert kvp.kvp_store_bytes_used(s) == per100
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put(s, 7, None, None, n_tokens=5)       # immutable: no overwrite
    assert e.value.code == kvp.KVP_E_EXISTS
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put(s, -1, None, None, n_tokens=5)
    assert e.value.code == kvp.KVP_E_INVAL
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put(s, 9, None, None, n_tokens=0)
    assert e.value.code == kvp.KVP_E_INVAL
    kvp.kvp_store_put(s, 9, None, None, n_tokens=200)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put(s, 10, None, None, n_tokens=1)
    assert e.value.code == kvp.KVP_E_NOSPACE
    assert kvp.kvp_store_bytes_used(s) == per100 + per200     # failed puts changed nothing
    assert kvp.kvp_store_packet_len(s, 10) == kvp.KVP_E_NOTFOUND


def _tiles(s):
    p = kvp.kvp_debug_last_plan(s, 0)
    n = int(p[0])
    return p[1:].reshape(n, 8)


def test_assemble_plan_offsets_and_tiles():
    s = dry_store()
    lens = {0: 72, 1: 1, 2: 64, 3: 130}
    for pid, n in lens.items():
        kvp.kvp_store_put(s, pid, None, None, n_tokens=n)
    cache = kvp.Cache.dry(2, t_cap=600)
    kvp.kvp_assemble(s, [([3, 1, 0, 3], 0), ([2], 10)], cache)
    assert list(cache.ctx_len[:2]) == [130 + 1 + 72 + 130, 74]
    t = _tiles(s)
    # request 0: Delta = 0, 130, 131, 203 (every adapter/document row occupies a position)
    want_pos = {0: [0, 130, 131, 203], 1: [10]}
    for r in (0, 1):
        rows = t[t[:, 6] == r]
        assert sorted(set(rows[:, 5])) == want_pos[r]
        covered = np.zeros(int(cache.ctx_len[r]), int)
        for src, stride, tok0, n_tok, dst, pos, _, _ in rows:
            assert 1 <= n_tok <= 64 and tok0 + n_tok <= stride
            assert dst == pos + tok0
            covered[dst:dst + n_tok] += 1
        base = 0 if r == 0 else 10
        assert np.all(covered[base:] == 1) and not covered[:base].any()
    # blobs are 256-byte aligned and disjoint
    starts = sorted(set(int(x) for x in t[:, 0]))
    assert all((x * 2) % 256 == 0 for x in starts)


def test_gather_tile_rows_follow_the_cache_layout_and_long_lists_plan():
    """Tiles hold up to 32 rows on a contiguous cache and up to 64 on a paged one; a list too long
    for the kernel arguments (more than 80 segments) plans the same way and covers every row once."""
    s = dry_store(max_positions=1 << 17)
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(1, 200, size=120)]
    for pid, n in enumerate(lens):
        kvp.kvp_store_put(s, pid, None, None, n_tokens=n)
    ids = list(range(120))
    total = sum(lens)
    contig = kvp.Cache.dry(1, t_cap=total)
    nb = (total + 15) // 16
    paged = kvp.Cache.dry(1, layout=kvp.KVP_PAGED, n_blocks=nb, block_size=16,
                          block_table=np.arange(nb, dtype=np.int32)[None, :])
    for cache, cap in ((contig, 32), (paged, 64)):
        kvp.kvp_assemble(s, [(ids, 0)], cache)
        t = _tiles(s)
        assert int(t[:, 3].max()) == cap
        covered = np.zeros(total, int)
        for src, stride, tok0, n_tok, dst, pos, _, _ in t:
            assert 1 <= n_tok <= cap and tok0 % cap == 0 and tok0 + n_tok <= stride and dst == pos + tok0
            covered[dst:dst + n_tok] += 1
        assert np.all(covered == 1)
        assert len(t) == sum((n + cap - 1) // cap for n in lens)


def test_empty_batches_are_legal_and_plan_nothing():
    s = dry_store()
    kvp.kvp_store_put(s, 0, None, None, n_tokens=50)
    cache = kvp.Cache.dry(1, t_cap=100)
    cache.ctx_len[0] = 7
    kvp.kvp_assemble(s, [], cache)
    assert int(kvp.kvp_debug_last_plan(s, 0)[0]) == 0 and cache.ctx_len[0] == 7
    none = np.array([0], np.int32)
    kvp.kvp_query_prefill(s, cache, 0, None, None, None, none, None, None)
    assert list(kvp.kvp_debug_last_plan(s, 1)[2:5]) == [0, 0, 0]      # no groups, items or slots
    kvp.kvp_prefill_packets(s, [], 0, None, None, None, none, None, None, None)
    assert list(kvp.kvp_debug_last_plan(s, 1)[2:5]) == [0, 0, 0]
    # a request without packets and without query rows is as empty
    kvp.kvp_assemble(s, [([], 0)], cache)
    assert cache.ctx_len[0] == 0 and int(kvp.kvp_debug_last_plan(s, 0)[0]) == 0
    kvp.kvp_query_prefill(s, cache, 0, None, None, None, np.array([0, 0], np.int32), None, None)
    assert list(kvp.kvp_debug_last_plan(s, 1)[2:5]) == [0, 0, 0]


def test_assemble_errors_leave_ctx_len_alone():
    s = dry_store(max_positions=300)
    kvp.kvp_store_put(s, 0, None, None, n_tokens=100)
    cache = kvp.Cache.dry(1, t_cap=150)
    cache.ctx_len[0] = -7
    for reqs, code in [([([5], 0)], kvp.KVP_E_NOTFOUND), ([([0, 0], 0)], kvp.KVP_E_CAPACITY),
                       ([([0], -1)], kvp.KVP_E_INVAL)]:
        with pytest.raises(kvp.KvpError) as e:
            kvp.kvp_assemble(s, reqs, cache)
        assert e.value.code == code and cache.ctx_len[0] == -7
    big = kvp.Cache.dry(1, t_cap=1000)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(s, [([0, 0, 0, 0], 0)], big)        # 400 rows > max_positions 300
    assert e.value.code == kvp.KVP_E_CAPACITY
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(s, [([0], 0)], big, layer_begin=1, layer_end=3)
    assert e.value.code == kvp.KVP_E_INVAL
    kvp.kvp_assemble(s, [([], 0)], big)                       # k = 0 is legal
    assert big.ctx_len[0] == 0 and len(_tiles(s)) == 0


def test_paged_block_table_is_validated():
    s = dry_store()
    kvp.kvp_store_put(s, 0, None, None, n_tokens=40)
    table = np.array([[3, 1, 2, 0]], np.int32)
    cache = kvp.Cache.dry(1, layout=kvp.KVP_PAGED, n_blocks=4, block_table=table)
    kvp.kvp_assemble(s, [([0], 0)], cache)
    assert cache.ctx_len[0] == 40
    with pytest.raises(kvp.KvpError) as e:                    # 80 rows need 5 blocks, table has 4
        kvp.kvp_assemble(s, [([0, 0], 0)], cache)
    assert e.value.code == kvp.KVP_E_CAPACITY
    bad = kvp.Cache.dry(1, layout=kvp.KVP_PAGED, n_blocks=4, block_table=np.array([[0, 9, 1, 2]], np.int32))
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(s, [([0], 0)], bad)
    assert e.value.code == kvp.KVP_E_INVAL
    odd = kvp.Cache.dry(1, layout=kvp.KVP_PAGED, n_blocks=4, block_table=table, block_size=12)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(s, [([0], 0)], odd)
    assert e.value.code == kvp.KVP_E_INVAL


def _attn_plan(s):
    p = kvp.kvp_debug_last_plan(s, 1)
    kind, bm, ng, ni, slots, need = (int(x) for x in p[:6])
    groups = p[6:6 + 6 * ng].reshape(ng, 6)
    items = p[6 + 6 * ng:].reshape(ni, 4)
    return kind, bm, groups, items, slots, need


def _random_prefill_cases(n):
    """Seeded random batch geometries: ragged contexts (some empty), ragged query counts (some
    zero), head groupings 1 / 4 / 7, both attention kernels."""
    rng = np.random.default_rng(4242)
    out = []
    for _ in range(n):
        n_kv = int(rng.choice([1, 2, 4, 8]))
        grp = int(rng.choice([1, 4, 7]))
        n_req = int(rng.integers(1, 9))
        big = rng.random() < 0.3
        ctx = [int(x) for x in rng.integers(0, 40000 if big else 3000, size=n_req)]
        n_q = [int(x) for x in rng.integers(0, 300, size=n_req)]
        if sum(n_q) == 0:
            n_q[0] = 1
        c = dict(n_q_heads=n_kv * grp, n_kv_heads=n_kv, ctx=ctx, n_q=n_q, max_positions=1 << 17)
        if rng.random() < 0.25:
            c.update(head_dim=64, dtype="f32")
        out.append(c)
    return out


@pytest.mark.parametrize("cfg", [
    dict(n_q_heads=32, n_kv_heads=8, ctx=[8192], n_q=[32]),
    dict(n_q_heads=28, n_kv_heads=4, ctx=[6720], n_q=[64]),
    dict(n_q_heads=32, n_kv_heads=8, ctx=[16896] * 8, n_q=[128] * 8),
    dict(n_q_heads=32, n_kv_heads=8, ctx=[0, 5, 1000, 77], n_q=[16, 0, 255, 1]),
    dict(n_q_heads=4, n_kv_heads=2, ctx=[144], n_q=[16], head_dim=64, dtype="f32"),
] + _random_prefill_cases(24))
def test_prefill_plan_covers_every_row_and_kv_exactly_once(cfg):
    cfg = dict(cfg)
    ctx, n_q = cfg.pop("ctx"), cfg.pop("n_q")
    s = dry_store(**cfg)
    g = s.cfg.n_q_heads // s.cfg.n_kv_heads
    n_req = len(ctx)
    cache = kvp.Cache.dry(n_req, t_cap=max(c + q for c, q in zip(ctx, n_q)))
    cache.ctx_len[:n_req] = ctx
    q_off = np.concatenate([[0], np.cumsum(n_q)]).astype(np.int32)
    kvp.kvp_query_prefill(s, cache, 0, None, None, None, q_off, None, None)
    kind, bm, groups, items, slots, need = _attn_plan(s)
    assert kind == (1 if (s.cfg.dtype == kvp.KVP_BF16 and s.cfg.head_dim == 128) else 0)
    seen = {}
    for gi, (r, h, m0, n_rows, part0, n_splits) in enumerate(groups):
        assert 1 <= n_rows <= bm and m0 % bm == 0
        rng = sorted((int(b), int(e)) for g_, sp, b, e in items if g_ == gi)
        assert len(rng) == n_splits
        t_last = (m0 + n_rows - 1) // g
        assert rng[0][0] == 0 and rng[-1][1] == ctx[r] + t_last + 1     # causal bound of the group
        for (b0, e0), (b1, e1) in zip(rng, rng[1:]):
            assert e0 == b1 and b0 < e0
        for m in range(m0, m0 + n_rows):
            assert (r, h, m) not in seen
            seen[(r, h, m)] = 1
    for r in range(n_req):
        for h in range(s.cfg.n_kv_heads):
            for m in range(n_q[r] * g):
                assert (r, h, m) in seen
    assert len(seen) == sum(n_q) * s.cfg.n_q_heads
    # split groups own disjoint partial slots; the workspace bound covers the need
    # (group gi owns slots gi * stride .., stride = the largest split count of the call)
    used = []
    stride = max([n_splits for *_, n_splits in groups if n_splits > 1] + [0])
    for gi, (r, h, m0, n_rows, part0, n_splits) in enumerate(groups):
        assert part0 == gi * stride
        if n_splits > 1:
            used += list(range(part0, part0 + n_splits))
    assert len(set(used)) == len(used) and all(0 <= u < slots for u in used)
    assert slots == len(groups) * stride
    bound = kvp.kvp_prefill_workspace_bytes(s, n_req, int(q_off[-1]), max(c + q for c, q in zip(ctx, n_q)))
    assert bound >= need


def test_paged_items_stay_within_the_block_id_limit(monkeypatch):
    """Paged layout: an item keeps its block ids in LDS, at most 2047 of them, so a long context
    is cut further than the work-item target asks for."""
    monkeypatch.setenv("KVP_ATTN_TARGET_ITEMS", "1")
    s = dry_store(n_q_heads=8, n_kv_heads=2, max_positions=1 << 17)
    ctx, n_q = [70000, 40000, 100], [8, 40, 3]
    n_blk = [(c + q + 15) // 16 for c, q in zip(ctx, n_q)]
    table = np.zeros((3, max(n_blk)), np.int32)
    at = 0
    for r in range(3):
        table[r, :n_blk[r]] = np.arange(at, at + n_blk[r])
        at += n_blk[r]
    cache = kvp.Cache.dry(3, layout=kvp.KVP_PAGED, n_blocks=at, block_table=table, block_size=16)
    cache.ctx_len[:3] = ctx
    q_off = np.concatenate([[0], np.cumsum(n_q)]).astype(np.int32)
    kvp.kvp_query_prefill(s, cache, 0, None, None, None, q_off, None, None)
    kind, bm, groups, items, slots, need = _attn_plan(s)
    assert kind == 1
    per_group = {}
    for g_, sp, b, e in items:
        if g_ < 0:                                             # padding of the launch order
            continue
        assert 0 < e - b <= 2047 * 16 and b % 64 == 0
        assert (e - 1) // 16 - b // 16 + 1 <= 2047             # block ids of the item
        per_group.setdefault(int(g_), []).append((int(b), int(e)))
    for gi, (r, h, m0, n_rows, part0, n_splits) in enumerate(groups):
        rng = sorted(per_group[gi])
        assert rng[0][0] == 0 and all(e0 == b1 for (_, e0), (b1, _) in zip(rng, rng[1:]))
        assert rng[-1][1] == ctx[r] + (m0 + n_rows - 1) // 4 + 1
        assert len(rng) == {0: 3, 1: 2, 2: 1}[int(r)]           # 70008 -> 3 ranges, 40040 -> 2, 103 -> 1
    assert kvp.kvp_prefill_workspace_bytes(s, 3, int(q_off[-1]), 70008) >= need


def test_prefill_errors():
    s = dry_store(max_positions=1000)
    cache = kvp.Cache.dry(1, t_cap=100)
    cache.ctx_len[0] = 90
    for q_off, code in [([0, 20], kvp.KVP_E_CAPACITY), ([1, 5], kvp.KVP_E_INVAL), ([0, -1], kvp.KVP_E_INVAL)]:
        with pytest.raises(kvp.KvpError) as e:
            kvp.kvp_query_prefill(s, cache, 0, None, None, None, np.array(q_off, np.int32), None, None)
        assert e.value.code == code
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_query_prefill(s, cache, 5, None, None, None, np.array([0, 4], np.int32), None, None)
    assert e.value.code == kvp.KVP_E_INVAL
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_query_prefill(s, cache, 0, None, None, None, np.array([0, 4], np.int32), None, None, flags=8)
    assert e.value.code == kvp.KVP_E_INVAL
    kvp.kvp_query_prefill(s, cache, 0, None, None, None, np.array([0, 10], np.int32), None, None)
    assert cache.ctx_len[0] == 90                             # prefill never advances ctx_len


def test_a_prefill_call_that_fails_on_its_workspace_keeps_the_kept_plans():
    import ctypes
    s = dry_store(max_positions=1 << 16)
    lib = kvp.load()
    cache = kvp.Cache.dry(1, t_cap=20000)

    def call(ctx, n_q, ws_bytes):
        cache.ctx_len[0] = ctx
        qo = np.array([0, n_q], np.int32)
        return lib.kvp_query_prefill(s.handle, ctypes.byref(cache.c), 0, None, None, None, qo.ctypes.data, 1, 0,
                                     None, ws_bytes, None, None)

    # fill the set of kept plans (max(8, n_layers + 1) entries), remember the last one's plan
    for i in range(8):
        assert call(1000 + 64 * i, 8, 1 << 60) == 0
    before = kvp.kvp_debug_last_plan(s, 1).copy()
    assert call(18000, 32, 4096) == kvp.KVP_E_CAPACITY             # a new geometry, workspace far too small
    assert "workspace" in kvp.kvp_last_error(s)
    assert np.array_equal(kvp.kvp_debug_last_plan(s, 1), before)   # nothing was planned into the store
    assert kvp.kvp_release_captured_plans(s) == 0                  # nothing was captured


def test_regular_one_request_plans_are_rebuilt_from_the_block_index():
    """A launch for one request whose packed rows fit one row block has a regular item pattern;
    its workgroups rebuild their items from their index, and the host only lets them after
    rebuilding every planned item with the same function.  Batches, several row blocks per head
    and the generic kernel keep reading their items from memory."""
    s = dry_store(n_q_heads=32, n_kv_heads=8, max_positions=1 << 17)
    for ctx, n_q, regular in [(8192, 32, True), (3000, 32, True), (8192, 1, True), (0, 20, True), (511, 30, True),
                              (100000, 7, True), (8192 - 32, 32, True), (6144 - 32, 32, True),   # (the last: 24 equal splits, none shorter)
                              (6720, 100, False), (100000, 200, False)]:
        cache = kvp.Cache.dry(1, t_cap=ctx + n_q)
        cache.ctx_len[0] = ctx
        kvp.kvp_query_prefill(s, cache, 0, None, None, None, np.array([0, n_q], np.int32), None, None)
        kind, bm, groups, items, slots, need = _attn_plan(s)
        assert kind == 1
        assert int(kvp.kvp_debug_last_plan(s, 2)[0]) == (len(items) if regular else 0), (ctx, n_q)
    cache = kvp.Cache.dry(2, t_cap=5000)
    cache.ctx_len[:2] = [4000, 3000]
    kvp.kvp_query_prefill(s, cache, 0, None, None, None, np.array([0, 32, 64], np.int32), None, None)
    assert int(kvp.kvp_debug_last_plan(s, 2)[0]) == 0                       # two requests
    f32 = dry_store(head_dim=64, dtype="f32")
    cache = kvp.Cache.dry(1, t_cap=600)
    cache.ctx_len[0] = 500
    kvp.kvp_query_prefill(f32, cache, 0, None, None, None, np.array([0, 5], np.int32), None, None)
    assert int(kvp.kvp_debug_last_plan(f32, 2)[0]) == 0                     # the generic kernel reads its items from memory


def test_packets_plan_tiles_and_items():
    s = dry_store(n_q_heads=32, n_kv_heads=8)
    lens = {0: 70, 1: 1, 2: 64, 3: 129}
    for pid, n in lens.items():
        kvp.kvp_store_put(s, pid, None, None, n_tokens=n)
    reqs = [([3, 1, 0], 0), ([], 0), ([2, 2], 0)]
    n_q = [40, 70, 0]
    q_off = np.concatenate([[0], np.cumsum(n_q)]).astype(np.int32)
    kvp.kvp_prefill_packets(s, reqs, 0, None, None, None, q_off, None, None, None)
    p = kvp.kvp_debug_last_plan(s, 1)
    kind, bm, ng, ni, slots, need = (int(x) for x in p[:6])
    assert kind == 2 and bm == 256                            # 70 query rows x 4 heads per kv head
    groups = p[6:6 + 6 * ng].reshape(ng, 6)
    items = p[6 + 6 * ng:6 + 6 * ng + 4 * ni].reshape(ni, 4)
    rest = p[6 + 6 * ng + 4 * ni:]
    tiles = rest[1:].reshape(int(rest[0]), 6)
    # request 0: packets 3, 1, 0 at Delta = 0, 129, 130, then one tile of query rows
    t0 = [tuple(int(v) for v in t[2:]) for t in tiles[:7]]
    assert t0 == [(0, 64, 0, 0), (64, 64, 0, 0), (128, 1, 0, 0), (0, 1, 129, 0), (0, 64, 130, 0), (64, 6, 130, 0),
                  (0, 40, 0, 1)]
    # request 1 has no packets: two tiles of query rows; request 2 has no query rows: no groups
    assert [tuple(int(v) for v in t[2:]) for t in tiles[7:9]] == [(0, 64, 0, 1), (64, 6, 0, 1)]
    assert set(int(x) for x in groups[:, 0]) == {0, 1}
    for gi, (r, h, m0, n_rows, part0, n_splits) in enumerate(groups):
        rng = sorted((int(b), int(e)) for g_, sp, b, e in items if g_ == gi)
        assert len(rng) == n_splits and all(e0 == b1 for (_, e0), (b1, _) in zip(rng, rng[1:]))
        first = 0 if r == 0 else 7
        t_last = (m0 + n_rows - 1) // 4
        n_pkt_tiles = 6 if r == 0 else 0
        assert rng[0][0] == first and rng[-1][1] == first + n_pkt_tiles + t_last // 64 + 1
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_prefill_packets(s, [([9], 0)], 0, None, None, None, np.array([0, 4], np.int32), None, None, None)
    assert e.value.code == kvp.KVP_E_NOTFOUND
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_prefill_packets(s, [([0], 3)], 0, None, None, None, np.array([0, 4], np.int32), None, None, None)
    assert e.value.code == kvp.KVP_E_INVAL
    f32 = dry_store(dtype="f32")
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_prefill_packets(f32, [([], 0)], 0, None, None, None, np.array([0, 4], np.int32), None, None, None)
    assert e.value.code == kvp.KVP_E_INVAL


def test_items_that_share_kv_rows_land_on_one_xcd():
    # config-4 geometry: 4 row blocks per (request, KV head); workgroup i runs on XCD i % 8
    s = dry_store(n_q_heads=32, n_kv_heads=8)
    n_req = 8
    cache = kvp.Cache.dry(n_req, t_cap=16896 + 128)
    cache.ctx_len[:n_req] = 16896
    q_off = (np.arange(n_req + 1) * 128).astype(np.int32)
    kvp.kvp_query_prefill(s, cache, 0, None, None, None, q_off, None, None)
    kind, bm, groups, items, slots, need = _attn_plan(s)
    where = {}
    for i, (gi, sp, b, e) in enumerate(items):
        if gi < 0:
            continue
        r, h = int(groups[gi][0]), int(groups[gi][1])
        where.setdefault((r, h, int(sp)), []).append(i)
    assert bm == 256 and len(where) * 2 == sum(len(v) for v in where.values())   # 512 packed rows / 256
    for idx in where.values():
        assert len({i % 8 for i in idx}) == 1            # one XCD
        assert max(idx) - min(idx) <= 24                 # adjacent in launch order


def test_compressed_packets_plan_rows_and_positions():
    """Sec. 5.4: positions advance by the packets' spans, rows by what each layer kept."""
    s = dry_store(n_layers=3)
    kvp.kvp_store_put(s, 0, None, None, n_tokens=40)                       # uncompressed
    kvp.kvp_store_put_compressed(s, 1, 100, None, None, n_rows=[100, 37, 0])  # 100 positions
    kvp.kvp_store_put_compressed(s, 2, 70, None, None, n_rows=[1, 70, 65])
    assert kvp.kvp_store_packet_len(s, 1) == 100
    assert [kvp.kvp_store_packet_rows(s, 1, l) for l in range(3)] == [100, 37, 0]
    assert kvp.kvp_store_packet_rows(s, 0, 2) == 40
    cache = kvp.Cache.dry(2, t_cap=400).with_ctx_rows(3)
    kvp.kvp_assemble(s, [([1, 0, 2], 5), ([0], 0)], cache)
    assert list(cache.ctx_len[:2]) == [5 + 100 + 40 + 70, 40]
    assert cache.ctx_rows[0].tolist() == [5 + 100 + 40 + 1, 5 + 37 + 40 + 70, 5 + 0 + 40 + 65]
    assert cache.ctx_rows[1].tolist() == [40, 40, 40]
    t = _tiles(s)
    # every tile of request 0 is rotated by the Delta of its packet: 5, 105, 145
    assert sorted(set(t[t[:, 6] == 0][:, 5])) == [5, 105, 145]
    # tiles of compressed packets carry a negative stride (their blob is laid out layer by layer)
    neg = t[t[:, 1] < 0]
    assert len(neg) and set(-neg[:, 1]) <= {100, 37, 1, 70, 65}
    # each tile names its layer; per (request, layer) the tiles cover the packet rows exactly once
    for r, base in ((0, 5), (1, 0)):
        for l in range(3):
            mine = t[(t[:, 6] == r) & (t[:, 7] == l)]
            rows = sorted(x for _, _, _, n, dst, *_ in mine for x in range(dst, dst + n))
            assert rows == list(range(base, int(cache.ctx_rows[r][l])))
    # a layer range writes only its own entries
    cache2 = kvp.Cache.dry(1, t_cap=400).with_ctx_rows(3)
    cache2.ctx_rows[:] = -1
    kvp.kvp_assemble(s, [([1], 0)], cache2, 1, 2)
    assert cache2.ctx_rows[0].tolist() == [-1, 37, -1] and cache2.ctx_len[0] == 100
    # the query side plans with the layer's rows and the request's position
    kvp.kvp_assemble(s, [([1, 0, 2], 5), ([0], 0)], cache)
    q_off = np.array([0, 4, 7], np.int32)
    kvp.kvp_query_prefill(s, cache, 1, None, None, None, q_off, None, None)
    kind, bm, groups, items, slots, need = _attn_plan(s)
    ends = {r: max(e for g_, sp, b, e in items if groups[g_][0] == r) for r in (0, 1)}
    assert ends[0] == cache.ctx_rows[0][1] + 4 and ends[1] == 40 + 3


def test_shared_header_plan_and_errors():
    """Sec. 4.1 (global adapters): header rows stored once; header-less packets get them back."""
    s = dry_store(n_layers=2, n_header=8)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_body(s, 0, None, None, n_tokens=100)          # no header yet
    assert e.value.code == kvp.KVP_E_INVAL
    kvp.kvp_store_put_header(s)
    used_header = kvp.kvp_store_bytes_used(s)
    assert used_header == kvp.packet_bytes(2, 2, 128, "bf16", 8)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_header(s)
    assert e.value.code == kvp.KVP_E_EXISTS
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_body(s, 0, None, None, n_tokens=8)            # nothing but the header
    assert e.value.code == kvp.KVP_E_INVAL
    kvp.kvp_store_put_body(s, 0, None, None, n_tokens=100)
    assert kvp.kvp_store_bytes_used(s) == used_header + kvp.packet_bytes(2, 2, 128, "bf16", 92)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_body(s, 0, None, None, n_tokens=50)
    assert e.value.code == kvp.KVP_E_EXISTS
    kvp.kvp_store_put(s, 1, None, None, n_tokens=40)                    # a whole packet next to it
    assert kvp.kvp_store_packet_len(s, 0) == 100 and kvp.kvp_store_packet_rows(s, 0, 1) == 100
    cache = kvp.Cache.dry(1, t_cap=300)
    kvp.kvp_assemble(s, [([0, 1, 0], 3)], cache)
    assert cache.ctx_len[0] == 3 + 100 + 40 + 100
    t = _tiles(s)
    covered = np.zeros(243, int)
    for src, stride, tok0, n_tok, dst, pos, _, _ in t:
        covered[dst:dst + n_tok] += 1
        assert pos in (3, 103, 143)
        if stride == 8:          # a header tile: from the shared blob, at the packet's first rows
            assert src * 2 < used_header and dst == pos and n_tok == 8 and pos in (3, 143)
        elif stride == 92:       # body rows land behind the header rows
            assert dst == pos + 8 + tok0
        else:
            assert stride == 40 and dst == pos + tok0
    assert np.all(covered[3:] == 1) and not covered[:3].any()
    assert sum(1 for row in t if row[1] == 8) == 2
    # the in-place path: a header tile of 8 rows, then the body tiles, all at the packet's Delta
    kvp.kvp_prefill_packets(s, [([0, 1], 0)], 0, None, None, None, np.array([0, 4], np.int32), None, None, None)
    p = kvp.kvp_debug_last_plan(s, 1)
    ng, ni = int(p[2]), int(p[3])
    rest = p[6 + 6 * ng + 4 * ni:]
    tiles = rest[1:].reshape(int(rest[0]), 6)
    assert [tuple(int(v) for v in x[1:]) for x in tiles] == [
        (8, 0, 8, 0, 0), (92, 0, 64, 0, 0), (92, 64, 28, 0, 0), (40, 0, 40, 100, 0), (0, 0, 4, 0, 1)]
    # a store without header rows has nothing to share
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_header(dry_store(n_header=0))
    assert e.value.code == kvp.KVP_E_INVAL


def test_compressed_packets_errors():
    s = dry_store(n_layers=2)
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_compressed(s, 0, 10, None, None, n_rows=[11, 3])
    assert e.value.code == kvp.KVP_E_INVAL
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_compressed(s, 0, 0, None, None, n_rows=[0, 0])
    assert e.value.code == kvp.KVP_E_INVAL
    kvp.kvp_store_put_compressed(s, 0, 10, None, None, n_rows=[10, 3])
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_store_put_compressed(s, 0, 10, None, None, n_rows=[1, 1])
    assert e.value.code == kvp.KVP_E_EXISTS
    cache = kvp.Cache.dry(1, t_cap=100)             # no ctx_rows
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(s, [([0], 0)], cache)
    assert e.value.code == kvp.KVP_E_INVAL and "ctx_rows" in str(e.value)
    cache = kvp.Cache.dry(1, t_cap=9).with_ctx_rows(2)   # layer 0 keeps 10 rows
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_assemble(s, [([0], 0)], cache)
    assert e.value.code == kvp.KVP_E_CAPACITY
    # the in-place attention path tiles the rows the called layer kept (packet 0: 10 and 3 rows),
    # at the positions of the spans
    kvp.kvp_store_put(s, 5, None, None, n_tokens=70)
    for layer, rows in ((0, 10), (1, 3)):
        kvp.kvp_prefill_packets(s, [([0, 5, 0], 0)], layer, None, None, None, np.array([0, 2], np.int32), None, None, None)
        p = kvp.kvp_debug_last_plan(s, 1)
        ng, ni = int(p[2]), int(p[3])
        rest = p[6 + 6 * ng + 4 * ni:]
        tiles = rest[1:].reshape(int(rest[0]), 6)
        assert [tuple(int(v) for v in x[1:]) for x in tiles] == [
            (-rows, 0, rows, 0, 0), (70, 0, 64, 10, 0), (70, 64, 6, 10, 0), (-rows, 0, rows, 80, 0), (0, 0, 2, 0, 1)]
        assert tiles[0][0] == tiles[3][0] and (layer == 0 or tiles[0][0] > 0)
    # rows of a layer cannot exceed the position
    cache = kvp.Cache.dry(1, t_cap=100).with_ctx_rows(2)
    cache.ctx_len[0] = 5
    cache.ctx_rows[0] = [6, 5]
    with pytest.raises(kvp.KvpError) as e:
        kvp.kvp_query_prefill(s, cache, 0, None, None, None, np.array([0, 1], np.int32), None, None)
    assert e.value.code == kvp.KVP_E_INVAL


def test_bench_refuses_more_than_one_gpu():
    # the build runs on one GPU; asking the benchmark for more ends with a message, no JSON line
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
