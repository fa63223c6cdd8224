"""ctypes binding of libkvp.so: the same entry points as include/kvp.h, taking torch
tensors for device memory.  Argument marshalling only -- every step of the path runs in
the library's HIP kernels.  There is no CPU fallback: if the library is missing, loading
fails.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvp.so")

KVP_F32, KVP_BF16 = 0, 1
KVP_CONTIG, KVP_PAGED = 0, 1
KVP_OK, KVP_E_INVAL, KVP_E_EXISTS, KVP_E_NOTFOUND = 0, -1, -2, -3
KVP_E_NOSPACE, KVP_E_CAPACITY, KVP_E_HIP = -4, -5, -6
KVP_PREROTATED = 1
KVP_DEVICE_NONE = -1

_vp, _i32, _i64, _u64, _u32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64,
                               ctypes.c_uint32)


class kvp_config_t(ctypes.Structure):
    _fields_ = [("n_layers", _i32), ("n_q_heads", _i32), ("n_kv_heads", _i32), ("head_dim", _i32),
                ("n_header", _i32), ("n_trailer", _i32), ("dtype", _i32), ("max_positions", _i32),
                ("rope_base", ctypes.c_double), ("inv_freq", _vp), ("arena", _vp),
                ("arena_bytes", _u64), ("device", _i32)]


class kvp_request_t(ctypes.Structure):
    _fields_ = [("packet_ids", _vp), ("k", _i32), ("base_pos", _i32)]


class kvp_cache_t(ctypes.Structure):
    _fields_ = [("layout", _i32), ("k", _vp), ("v", _vp), ("t_cap", _i32), ("n_blocks", _i32),
                ("block_size", _i32), ("block_table", _vp), ("max_blocks_per_req", _i32),
                ("ctx_len", _vp), ("ctx_rows", _vp)]


EXPORTS = {
    "kvp_store_create": (_i32, [ctypes.POINTER(kvp_config_t), ctypes.POINTER(_vp)]),
    "kvp_store_destroy": (_i32, [_vp]),
    "kvp_store_put": (_i32, [_vp, _i64, _i32, _vp, _vp, _i32, _vp]),
    "kvp_store_put_compressed": (_i32, [_vp, _i64, _i32, _vp, _vp, _vp, _i32, _vp]),
    "kvp_store_put_header": (_i32, [_vp, _vp, _vp, _i32, _vp]),
    "kvp_store_put_body": (_i32, [_vp, _i64, _i32, _vp, _vp, _i32, _vp]),
    "kvp_store_packet_len": (_i32, [_vp, _i64]),
    "kvp_store_packet_rows": (_i32, [_vp, _i64, _i32]),
    "kvp_store_bytes_used": (_u64, [_vp]),
    "kvp_store_arena_on_host": (_i32, [_vp]),
    "kvp_packet_bytes": (_u64, [ctypes.POINTER(kvp_config_t), _i32]),
    "kvp_assemble": (_i32, [_vp, ctypes.POINTER(kvp_request_t), _i32, _i32, _i32,
                            ctypes.POINTER(kvp_cache_t), _vp]),
    "kvp_query_prefill": (_i32, [_vp, ctypes.POINTER(kvp_cache_t), _i32, _vp, _vp, _vp, _vp, _i32,
                                 _u32, _vp, _u64, _vp, _vp]),
    "kvp_prefill_packets": (_i32, [_vp, ctypes.POINTER(kvp_request_t), _i32, _i32, _vp, _vp, _vp, _vp, _u32,
                                   _vp, _vp, _u64, _vp, _vp]),
    "kvp_query_prefill_static": (_i32, [_vp, ctypes.POINTER(kvp_cache_t), _i32, _vp, _vp, _vp, _vp, _i32,
                                        _u32, _vp, _vp]),
    "kvp_static_workspace_bytes": (_u64, []),
    "kvp_release_captured_plans": (_i32, [_vp]),
    "kvp_prefill_workspace_bytes": (_u64, [_vp, _i32, _i32, _i32]),
    "kvp_last_error": (ctypes.c_char_p, [_vp]),
    "kvp_debug_last_plan": (_i64, [_vp, _i32, _vp, _i64]),
    "kvp_version": (ctypes.c_char_p, []),
}

_lib = None


def load():
    """Loads libkvp.so (built by paper_2604_13226_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libkvp.so is not built: run `python -m paper_2604_13226_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


class KvpError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("kvp error %d: %s" % (code, text))
        self.code = code


def _check(store, rc):
    if rc != 0:
        raise KvpError(rc, (load().kvp_last_error(store) or b"").decode())


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)  # the current stream's handle without a Stream object


def _stream(stream, store=None):
    """Raw hipStream_t of `stream` (a torch stream or a raw handle), or of torch's current stream
    on the store's device."""
    if stream is None:
        if store is not None:
            if store.dry:
                return None
            if _raw_stream is not None:
                return _raw_stream(store.cfg.device)
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def _dtype_code(dt):
    return {torch.float32: KVP_F32, torch.bfloat16: KVP_BF16, "f32": KVP_F32, "bf16": KVP_BF16}[dt]


class Store:
    """Handle of a kvp_store_t plus the arena tensor it points into (the caller's memory)."""

    def __init__(self, handle, cfg, arena):
        self.handle, self.cfg, self.arena = handle, cfg, arena
        self.dry = cfg.device == KVP_DEVICE_NONE
        self.torch_dtype = torch.bfloat16 if cfg.dtype == KVP_BF16 else torch.float32
        self.q_row = (cfg.n_q_heads, cfg.head_dim)     # trailing dims of q / out
        self.kv_row = (cfg.n_kv_heads, cfg.head_dim)   # ... of k_new / v_new

    def __del__(self):
        try:
            kvp_store_destroy(self)
        except Exception:
            pass


def kvp_store_create(n_layers, n_q_heads, n_kv_heads, head_dim, dtype, rope_base, max_positions,
                     arena_bytes, n_header=0, n_trailer=0, device=0, inv_freq=None, arena="device"):
    """kvp_store_create: allocates the arena with torch (on `device`, or with arena="host" in
    pinned host memory) and creates the store.  device=KVP_DEVICE_NONE makes a planning-only
    store (no GPU touched)."""
    L = load()
    cfg = kvp_config_t()
    cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = n_layers, n_q_heads, n_kv_heads, head_dim
    cfg.n_header, cfg.n_trailer = n_header, n_trailer
    cfg.dtype = _dtype_code(dtype)
    cfg.max_positions = max_positions
    cfg.rope_base = float(rope_base)
    keep = None
    if inv_freq is not None:
        keep = np.ascontiguousarray(inv_freq, np.float32)
        cfg.inv_freq = keep.ctypes.data
    where, arena = arena, None
    if device != KVP_DEVICE_NONE:
        if where == "host":
            arena = torch.empty(int(arena_bytes) + 256, dtype=torch.uint8, pin_memory=True)
        else:
            assert where == "device", where
            arena = torch.empty(int(arena_bytes) + 256, dtype=torch.uint8, device="cuda:%d" % device)
        base = (arena.data_ptr() + 255) // 256 * 256
        cfg.arena = base
    cfg.arena_bytes = int(arena_bytes)
    cfg.device = device
    h = _vp()
    rc = L.kvp_store_create(ctypes.byref(cfg), ctypes.byref(h))
    if rc != 0:
        raise KvpError(rc, (L.kvp_last_error(None) or b"").decode())
    return Store(h, cfg, arena)


def kvp_store_destroy(store):
    if store.handle is not None:
        h, store.handle = store.handle, None
        load().kvp_store_destroy(h)


def kvp_store_put(store, packet_id, k, v, stream=None, n_tokens=None):
    """k, v: torch tensors [n_layers][n_kv_heads][n_tokens][head_dim] on the GPU or the CPU."""
    if store.dry:
        rc = load().kvp_store_put(store.handle, int(packet_id), int(n_tokens), None, None, 0, None)
        return _check(store.handle, rc)
    assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
    assert k.dtype == store.torch_dtype and v.dtype == store.torch_dtype
    c = store.cfg
    assert tuple(k.shape[:2]) == (c.n_layers, c.n_kv_heads) and k.shape[3] == c.head_dim
    on_dev = 1 if k.is_cuda else 0
    assert v.is_cuda == k.is_cuda
    rc = load().kvp_store_put(store.handle, int(packet_id), int(k.shape[2]), k.data_ptr(), v.data_ptr(),
                              on_dev, _stream(stream))
    _check(store.handle, rc)


def kvp_store_put_compressed(store, packet_id, span, k_layers, v_layers, stream=None, n_rows=None):
    """A compressed packet: k_layers[l], v_layers[l] are torch tensors [n_kv_heads][rows_l][head_dim]
    (the rows layer l kept), all on the GPU or all on the CPU; span = the positions it occupies."""
    c = store.cfg
    if store.dry:
        rows = np.ascontiguousarray(n_rows, np.int32)
        rc = load().kvp_store_put_compressed(store.handle, int(packet_id), int(span), rows.ctypes.data,
                                             None, None, 0, None)
        return _check(store.handle, rc)
    assert len(k_layers) == c.n_layers == len(v_layers)
    rows = np.array([int(k.shape[1]) for k in k_layers], np.int32)
    for k, v in zip(k_layers, v_layers):
        assert k.shape == v.shape and k.shape[0] == c.n_kv_heads and k.shape[2] == c.head_dim
        assert k.dtype == store.torch_dtype and v.dtype == store.torch_dtype
    kk = torch.cat([k.reshape(-1) for k in k_layers]).contiguous()
    vv = torch.cat([v.reshape(-1) for v in v_layers]).contiguous()
    rc = load().kvp_store_put_compressed(store.handle, int(packet_id), int(span), rows.ctypes.data,
                                         kk.data_ptr(), vv.data_ptr(), 1 if kk.is_cuda else 0, _stream(stream))
    if kk.is_cuda:
        torch.cuda.synchronize()  # kk, vv are temporaries
    _check(store.handle, rc)


def kvp_store_put_header(store, k=None, v=None, stream=None):
    """The header rows every packet starts with, stored once: k, v [n_layers][n_kv_heads][n_header][head_dim]."""
    if store.dry:
        return _check(store.handle, load().kvp_store_put_header(store.handle, None, None, 0, None))
    c = store.cfg
    assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
    assert k.dtype == store.torch_dtype and v.dtype == store.torch_dtype and v.is_cuda == k.is_cuda
    assert tuple(k.shape) == (c.n_layers, c.n_kv_heads, c.n_header, c.head_dim)
    rc = load().kvp_store_put_header(store.handle, k.data_ptr(), v.data_ptr(), 1 if k.is_cuda else 0, _stream(stream))
    _check(store.handle, rc)


def kvp_store_put_body(store, packet_id, k, v, stream=None, n_tokens=None):
    """A packet without its header rows: k, v [n_layers][n_kv_heads][n_tokens - n_header][head_dim]
    (rows n_header.. of the packet); n_tokens, header included, is derived from the shape."""
    if store.dry:
        rc = load().kvp_store_put_body(store.handle, int(packet_id), int(n_tokens), None, None, 0, None)
        return _check(store.handle, rc)
    c = store.cfg
    assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
    assert k.dtype == store.torch_dtype and v.dtype == store.torch_dtype and v.is_cuda == k.is_cuda
    assert tuple(k.shape[:2]) == (c.n_layers, c.n_kv_heads) and k.shape[3] == c.head_dim
    rc = load().kvp_store_put_body(store.handle, int(packet_id), int(k.shape[2]) + c.n_header, k.data_ptr(),
                                   v.data_ptr(), 1 if k.is_cuda else 0, _stream(stream))
    _check(store.handle, rc)


def kvp_store_packet_len(store, packet_id):
    return int(load().kvp_store_packet_len(store.handle, int(packet_id)))


def kvp_store_packet_rows(store, packet_id, layer):
    return int(load().kvp_store_packet_rows(store.handle, int(packet_id), int(layer)))


def kvp_store_bytes_used(store):
    return int(load().kvp_store_bytes_used(store.handle))


def kvp_store_arena_on_host(store):
    return int(load().kvp_store_arena_on_host(store.handle))


def kvp_packet_bytes(store, n_tokens):
    return int(load().kvp_packet_bytes(ctypes.byref(store.cfg), int(n_tokens)))


def packet_bytes(n_layers, n_kv_heads, head_dim, dtype, n_tokens):
    """kvp_packet_bytes for a configuration not yet turned into a store (to size an arena)."""
    cfg = kvp_config_t()
    cfg.n_layers, cfg.n_kv_heads, cfg.head_dim, cfg.dtype = n_layers, n_kv_heads, head_dim, _dtype_code(dtype)
    return int(load().kvp_packet_bytes(ctypes.byref(cfg), int(n_tokens)))


class Cache:
    """kvp_cache_t plus the tensors/arrays it points to.

    CONTIG: k, v [n_req][n_layers][n_kv_heads][t_cap][d].
    PAGED : k, v pools [n_layers][n_blocks][n_kv_heads][block_size][d]; block_table is a
            host int32 array [n_req][max_blocks_per_req].
    """

    def __init__(self, k, v, n_req, layout=KVP_CONTIG, block_table=None, block_size=16):
        self.k, self.v, self.n_req, self.layout = k, v, n_req, layout
        self.ctx_len = np.zeros(max(n_req, 1), np.int32)
        self.block_table = None
        c = kvp_cache_t()
        c.layout = layout
        c.k = k.data_ptr() if k is not None else None
        c.v = v.data_ptr() if v is not None else None
        if layout == KVP_CONTIG:
            c.t_cap = int(k.shape[3])
        else:
            self.block_table = np.ascontiguousarray(block_table, np.int32)
            assert self.block_table.ndim == 2 and self.block_table.shape[0] == n_req
            c.n_blocks = int(k.shape[1])
            c.block_size = int(block_size)
            c.block_table = self.block_table.ctypes.data
            c.max_blocks_per_req = int(self.block_table.shape[1])
        c.ctx_len = self.ctx_len.ctypes.data
        self.ctx_rows = None
        self.c = c

    def with_ctx_rows(self, n_layers):
        """Adds the per-layer row counts (kvp_cache_t.ctx_rows) that compressed packets need."""
        self.ctx_rows = np.zeros((max(self.n_req, 1), n_layers), np.int32)
        self.c.ctx_rows = self.ctx_rows.ctypes.data
        return self

    @staticmethod
    def contiguous(store, n_req, t_cap, device="cuda:0"):
        g = store.cfg
        shape = (n_req, g.n_layers, g.n_kv_heads, t_cap, g.head_dim)
        k = torch.zeros(shape, dtype=store.torch_dtype, device=device)
        v = torch.zeros(shape, dtype=store.torch_dtype, device=device)
        return Cache(k, v, n_req)

    @staticmethod
    def dry(n_req, t_cap=0, layout=KVP_CONTIG, n_blocks=0, block_table=None, block_size=16):
        """Cache descriptor without device memory, for planning-only stores."""
        class _Fake:
            def __init__(self, shape): self.shape = shape
            def data_ptr(self): return 4096
        if layout == KVP_CONTIG:
            f = _Fake((n_req, 0, 0, t_cap, 0))
            return Cache(f, f, n_req)
        f = _Fake((0, n_blocks, 0, block_size, 0))
        return Cache(f, f, n_req, KVP_PAGED, block_table, block_size)

    @staticmethod
    def paged(store, n_req, n_blocks, block_table, block_size=16, device="cuda:0"):
        g = store.cfg
        shape = (g.n_layers, n_blocks, g.n_kv_heads, block_size, g.head_dim)
        k = torch.zeros(shape, dtype=store.torch_dtype, device=device)
        v = torch.zeros(shape, dtype=store.torch_dtype, device=device)
        return Cache(k, v, n_req, KVP_PAGED, block_table, block_size)

    def logical(self, r, layer, n_rows):
        """(K, V) rows 0..n_rows-1 of request r at `layer` as [n_kv_heads][n_rows][d] tensors."""
        if self.layout == KVP_CONTIG:
            return self.k[r, layer, :, :n_rows], self.v[r, layer, :, :n_rows]
        bs = self.c.block_size
        nb = (n_rows + bs - 1) // bs
        blocks = torch.as_tensor(self.block_table[r, :nb].astype(np.int64), device=self.k.device)
        def gather(pool):
            x = pool[layer, blocks]                       # [nb][Hkv][bs][d]
            x = x.permute(1, 0, 2, 3).reshape(pool.shape[2], nb * bs, pool.shape[4])
            return x[:, :n_rows]
        return gather(self.k), gather(self.v)


def _requests(requests):
    n_req = len(requests)
    arr = (kvp_request_t * max(n_req, 1))()
    keep = []
    for i, (ids, base_pos) in enumerate(requests):
        a = np.ascontiguousarray(ids, np.int64)
        keep.append(a)
        arr[i].packet_ids = a.ctypes.data if len(a) else None
        arr[i].k = len(a)
        arr[i].base_pos = int(base_pos)
    return arr, keep


def kvp_assemble(store, requests, cache, layer_begin=0, layer_end=None, stream=None):
    """requests: list of (packet_ids, base_pos).  Fills cache.ctx_len."""
    n_req = len(requests)
    arr, keep = _requests(requests)
    if layer_end is None:
        layer_end = store.cfg.n_layers
    rc = load().kvp_assemble(store.handle, arr, n_req, int(layer_begin), int(layer_end),
                             ctypes.byref(cache.c), _stream(stream, store))
    if rc:
        _check(store.handle, rc)


def kvp_prefill_workspace_bytes(store, n_req, max_tot_q, max_ctx):
    return int(load().kvp_prefill_workspace_bytes(store.handle, int(n_req), int(max_tot_q), int(max_ctx)))


def _check_qkv(store, tot_q, q, k_new, v_new, out, k_tail=None):
    """The kernels take these shapes for granted: dense device tensors of the store's dtype,
    [tot_q][heads][head_dim]."""
    td = store.torch_dtype
    qs, ks = (tot_q,) + store.q_row, (tot_q,) + store.kv_row
    ok = (q.shape == qs and out.shape == qs and k_new.shape == ks and v_new.shape == ks
          and q.dtype == td and out.dtype == td and k_new.dtype == td and v_new.dtype == td
          and q.is_cuda and out.is_cuda and k_new.is_cuda and v_new.is_cuda
          and q.is_contiguous() and out.is_contiguous() and k_new.is_contiguous() and v_new.is_contiguous())
    if k_tail is not None:
        ok = ok and k_tail.shape == ks and k_tail.dtype == td and k_tail.is_cuda and k_tail.is_contiguous()
    if not ok:
        raise ValueError("q / out must be dense %s tensors on the GPU of shape %s, k_new / v_new%s of shape %s"
                         % (td, qs, " / k_tail" if k_tail is not None else "", ks))


def kvp_query_prefill(store, cache, layer, q, k_new, v_new, q_offsets, workspace, out, flags=0,
                      stream=None):
    """q [tot_q][Hq][d], k_new/v_new [tot_q][Hkv][d], out like q: torch tensors on the GPU;
    q_offsets: host int32 [n_req+1]; workspace: torch uint8 tensor, 256-byte aligned."""
    qo = np.ascontiguousarray(q_offsets, np.int32)
    n_req = len(qo) - 1
    if store.dry:
        rc = load().kvp_query_prefill(store.handle, ctypes.byref(cache.c), int(layer), None, None, None,
                                      qo.ctypes.data, n_req, int(flags), None, 1 << 60, None, None)
        return _check(store.handle, rc)
    _check_qkv(store, int(qo[-1]), q, k_new, v_new, out)
    rc = load().kvp_query_prefill(store.handle, ctypes.byref(cache.c), int(layer), q.data_ptr(),
                                  k_new.data_ptr(), v_new.data_ptr(), qo.ctypes.data, n_req, int(flags),
                                  workspace.data_ptr(), workspace.numel(), out.data_ptr(),
                                  _stream(stream, store))
    if rc:
        _check(store.handle, rc)


def kvp_query_prefill_static(store, cache, layer, q, k_new, v_new, q_offsets, out, flags=0, stream=None):
    """kvp_query_prefill without a workspace argument: scratch and plan live in the library's
    static device array (the entry point that allocates nothing)."""
    qo = np.ascontiguousarray(q_offsets, np.int32)
    n_req = len(qo) - 1
    _check_qkv(store, int(qo[-1]), q, k_new, v_new, out)
    rc = load().kvp_query_prefill_static(store.handle, ctypes.byref(cache.c), int(layer), q.data_ptr(),
                                         k_new.data_ptr(), v_new.data_ptr(), qo.ctypes.data, n_req, int(flags),
                                         out.data_ptr(), _stream(stream, store))
    if rc:
        _check(store.handle, rc)


def kvp_static_workspace_bytes():
    return int(load().kvp_static_workspace_bytes())


def kvp_prefill_packets(store, requests, layer, q, k_new, v_new, q_offsets, k_tail, workspace, out,
                        flags=0, stream=None):
    """Attention of the query rows over the requests' packets read in place from the store.
    requests: list of (packet_ids, 0); k_tail [tot_q][Hkv][d] receives the rotated K_new."""
    qo = np.ascontiguousarray(q_offsets, np.int32)
    n_req = len(qo) - 1
    arr, keep = _requests(requests)
    if store.dry:
        rc = load().kvp_prefill_packets(store.handle, arr, n_req, int(layer), None, None, None, qo.ctypes.data,
                                        int(flags), None, None, 1 << 60, None, None)
        return _check(store.handle, rc)
    _check_qkv(store, int(qo[-1]), q, k_new, v_new, out, k_tail)
    rc = load().kvp_prefill_packets(store.handle, arr, n_req, int(layer), q.data_ptr(), k_new.data_ptr(),
                                    v_new.data_ptr(), qo.ctypes.data, int(flags), k_tail.data_ptr(),
                                    workspace.data_ptr(), workspace.numel(), out.data_ptr(),
                                    _stream(stream, store))
    if rc:
        _check(store.handle, rc)


def kvp_release_captured_plans(store):
    """Makes the plans kept for destroyed HIP graphs replaceable again; returns how many."""
    return int(load().kvp_release_captured_plans(store.handle))


def kvp_last_error(store):
    return (load().kvp_last_error(store.handle if store else None) or b"").decode()


def kvp_debug_last_plan(store, which):
    n = int(load().kvp_debug_last_plan(store.handle, int(which), None, 0))
    out = np.zeros(max(n, 1), np.int64)
    load().kvp_debug_last_plan(store.handle, int(which), out.ctypes.data, n)
    return out[:n]


def kvp_version():
    return load().kvp_version().decode()


def alloc_workspace(nbytes, device="cuda:0"):
    """256-byte aligned uint8 workspace tensor of at least nbytes."""
    t = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=device)
    off = (-t.data_ptr()) % 256
    return t[off:off + int(nbytes)]
