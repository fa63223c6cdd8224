"""ctypes front end of the CPU oracle (kvp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  Nothing here touches the HIP library, and the
HIP library never touches this.

Arrays are numpy.  bf16 tensors travel as ``uint16`` bit patterns, fp32 as
``float32``; ``dtype`` is "f32" or "bf16".
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvp_oracle.c")
_LIB = os.path.join(_HERE, "libkvp_oracle.so")

F32, BF16 = 0, 1
_DT = {"f32": F32, "bf16": BF16}
_NP = {"f32": np.float32, "bf16": np.uint16}


def build(force=False):
    """Compile kvp_oracle.c with gcc (no FMA contraction, OpenMP)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        # tests/test_oracle_mutants.py points the pins at deliberately broken copies of the oracle
        # to show that they notice.  Another library is taken only when that test says it is the
        # one asking (a second variable), never on a GPU machine's parity run by accident, and the
        # substitution is announced.
        path = None
        if os.environ.get("KVP_ORACLE_LIB") and os.environ.get("KVP_ORACLE_LIB_FOR") == "tests/test_oracle_mutants.py":
            path = os.environ["KVP_ORACLE_LIB"]
            import sys
            print("oracle: using the substituted library %s" % path, file=sys.stderr, flush=True)
        path = path or build()
        L = ctypes.CDLL(path)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        L.kvo_inv_freq.argtypes = [dbl, i32, vp]
        L.kvo_inv_freq.restype = None
        L.kvo_cos_sin.argtypes = [i64, vp, i32, vp, vp]
        L.kvo_cos_sin.restype = None
        L.kvo_rotate.argtypes = [vp, i32, vp, vp, vp]
        L.kvo_rotate.restype = None
        L.kvo_assemble.argtypes = [i32, i32, i32, i32, vp, i32, vp, vp, vp, i64, i64, vp, vp]
        L.kvo_assemble.restype = i64
        L.kvo_query_rope_append.argtypes = [i32, i32, i32, i32, vp, i32, i64, vp, vp, vp,
                                            i32, vp, vp, i64, vp]
        L.kvo_query_rope_append.restype = None
        L.kvo_attention.argtypes = [i32, i32, i32, i32, i32, i64, vp, vp, vp, i64, vp]
        L.kvo_attention.restype = None
        L.kvo_assemble_layer_spans.argtypes = [i32, i32, i32, vp, i32, vp, vp, vp, vp, i64, i64, vp, vp, vp]
        L.kvo_assemble_layer_spans.restype = i64
        L.kvo_query_rope_append_at.argtypes = [i32, i32, i32, i32, vp, i32, i64, i64, vp, vp, vp,
                                               i32, vp, vp, i64, vp]
        L.kvo_query_rope_append_at.restype = None
        L.kvo_num_threads.argtypes = []
        L.kvo_num_threads.restype = i32
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, shape=None):
    a = np.ascontiguousarray(a)
    assert a.dtype == _NP[dtype], (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def num_threads():
    return int(lib().kvo_num_threads())


def inv_freq(rope_base, d):
    """theta_i = base^(-2i/d) as fp32, i < d/2."""
    out = np.empty(d // 2, np.float32)
    lib().kvo_inv_freq(float(rope_base), d, _p(out))
    return out


def cos_sin(pos, inv_f):
    inv_f = _chk(inv_f, "f32")
    d = 2 * inv_f.shape[0]
    c = np.empty(d // 2, np.float32)
    s = np.empty(d // 2, np.float32)
    lib().kvo_cos_sin(int(pos), _p(inv_f), d, _p(c), _p(s))
    return c, s


def rotate(x, pos, inv_f):
    """Eq. 1 applied to one fp32 head vector: R_{Theta,pos} x."""
    x = _chk(x, "f32")
    d = x.shape[0]
    c, s = cos_sin(pos, inv_f)
    y = np.empty(d, np.float32)
    lib().kvo_rotate(_p(x), d, _p(c), _p(s), _p(y))
    return y


def assemble(dtype, packets_k, packets_v, inv_f, base_pos=0, t_cap=None, k_out=None, v_out=None):
    """Realign + concatenate packets for one request.

    packets_k/v: lists of arrays [n_layers][n_kv][len_j][d].
    Returns (k_cache, v_cache, ctx_len), caches [n_layers][n_kv][t_cap][d].
    """
    inv_f = _chk(inv_f, "f32")
    k = len(packets_k)
    d = 2 * inv_f.shape[0]
    lens = np.array([p.shape[2] for p in packets_k], np.int32)
    total = int(base_pos + lens.sum())
    if k:
        n_layers, n_kv = packets_k[0].shape[:2]
    else:
        assert k_out is not None
        n_layers, n_kv = k_out.shape[:2]
    if t_cap is None:
        t_cap = total if k_out is None else k_out.shape[2]
    pk = [_chk(p, dtype, (n_layers, n_kv, int(l), d)) for p, l in zip(packets_k, lens)]
    pv = [_chk(p, dtype, (n_layers, n_kv, int(l), d)) for p, l in zip(packets_v, lens)]
    if k_out is None:
        k_out = np.zeros((n_layers, n_kv, t_cap, d), _NP[dtype])
        v_out = np.zeros((n_layers, n_kv, t_cap, d), _NP[dtype])
    assert k_out.flags.c_contiguous and v_out.flags.c_contiguous
    assert k_out.shape == (n_layers, n_kv, t_cap, d) and k_out.dtype == _NP[dtype]
    arr_t = ctypes.c_void_p * max(k, 1)
    ak = arr_t(*[p.ctypes.data for p in pk]) if k else arr_t()
    av = arr_t(*[p.ctypes.data for p in pv]) if k else arr_t()
    r = lib().kvo_assemble(_DT[dtype], n_layers, n_kv, d, _p(inv_f), k,
                           ctypes.cast(ak, ctypes.c_void_p), ctypes.cast(av, ctypes.c_void_p),
                           _p(lens), int(base_pos), int(t_cap), _p(k_out), _p(v_out))
    if r < 0:
        raise ValueError("context does not fit t_cap")
    return k_out, v_out, int(r)


def query_rope_append(dtype, q, k_new, v_new, inv_f, ctx_len, k_layer, v_layer, prerotated=False):
    """Rotate Q/K_new to rows ctx_len+t, append K_new/V_new in place.

    q [n_q][Hq][d]; k_new, v_new [n_q][Hkv][d]; k_layer, v_layer [Hkv][t_cap][d].
    Returns the rotated query, fp32 [n_q][Hq][d].
    """
    inv_f = _chk(inv_f, "f32")
    q = _chk(q, dtype)
    n_q, n_q_heads, d = q.shape
    n_kv, t_cap, _ = k_layer.shape
    k_new = _chk(k_new, dtype, (n_q, n_kv, d))
    v_new = _chk(v_new, dtype, (n_q, n_kv, d))
    assert k_layer.flags.c_contiguous and v_layer.flags.c_contiguous
    assert k_layer.dtype == _NP[dtype] and v_layer.dtype == _NP[dtype]
    assert ctx_len + n_q <= t_cap
    q_rot = np.empty((n_q, n_q_heads, d), np.float32)
    lib().kvo_query_rope_append(_DT[dtype], n_q_heads, n_kv, d, _p(inv_f), n_q, int(ctx_len),
                                _p(q), _p(k_new), _p(v_new), int(bool(prerotated)),
                                _p(k_layer), _p(v_layer), int(t_cap), _p(q_rot))
    return q_rot


def assemble_layer_spans(dtype, packets_k, packets_v, spans, inv_f, base_pos=0, t_cap=None):
    """One layer of a cache composed of compressed packets (Sec. 5.4).

    packets_k/v: lists of arrays [n_kv][rows_j][d] (the rows packet j kept in this layer);
    spans[j]: positions packet j occupies.  Returns (k_layer, v_layer, n_rows, pos_end),
    layers [n_kv][t_cap][d]."""
    inv_f = _chk(inv_f, "f32")
    k = len(packets_k)
    assert k >= 1 and len(spans) == k
    d = 2 * inv_f.shape[0]
    rows = np.array([p.shape[1] for p in packets_k], np.int32)
    spans = np.ascontiguousarray(spans, np.int32)
    n_kv = packets_k[0].shape[0]
    if t_cap is None:
        t_cap = int(rows.sum())
    pk = [_chk(p, dtype, (n_kv, int(r), d)) for p, r in zip(packets_k, rows)]
    pv = [_chk(p, dtype, (n_kv, int(r), d)) for p, r in zip(packets_v, rows)]
    k_out = np.zeros((n_kv, t_cap, d), _NP[dtype])
    v_out = np.zeros((n_kv, t_cap, d), _NP[dtype])
    arr_t = ctypes.c_void_p * k
    ak, av = arr_t(*[p.ctypes.data for p in pk]), arr_t(*[p.ctypes.data for p in pv])
    pos_end = np.zeros(1, np.int64)
    r = lib().kvo_assemble_layer_spans(_DT[dtype], n_kv, d, _p(inv_f), k, ctypes.cast(ak, ctypes.c_void_p),
                                       ctypes.cast(av, ctypes.c_void_p), _p(rows), _p(spans), int(base_pos),
                                       int(t_cap), _p(k_out), _p(v_out), _p(pos_end))
    if r < 0:
        raise ValueError("rows do not fit t_cap")
    return k_out, v_out, int(r), int(pos_end[0])


def query_prefill_at(dtype, q, k_new, v_new, inv_f, row0, pos0, k_layer, v_layer, prerotated=False):
    """One layer of the query side when rows and positions differ: the query tokens sit at
    positions pos0 + t, their K/V go to cache rows row0 + t; then attention over rows
    0 .. row0 + t."""
    inv_f = _chk(inv_f, "f32")
    q = _chk(q, dtype)
    n_q, n_q_heads, d = q.shape
    n_kv, t_cap, _ = k_layer.shape
    k_new = _chk(k_new, dtype, (n_q, n_kv, d))
    v_new = _chk(v_new, dtype, (n_q, n_kv, d))
    assert k_layer.flags.c_contiguous and v_layer.flags.c_contiguous
    assert k_layer.dtype == _NP[dtype] and v_layer.dtype == _NP[dtype]
    assert row0 + n_q <= t_cap
    q_rot = np.empty((n_q, n_q_heads, d), np.float32)
    lib().kvo_query_rope_append_at(_DT[dtype], n_q_heads, n_kv, d, _p(inv_f), n_q, int(row0), int(pos0),
                                   _p(q), _p(k_new), _p(v_new), int(bool(prerotated)),
                                   _p(k_layer), _p(v_layer), int(t_cap), _p(q_rot))
    return attention(dtype, q_rot, k_layer, v_layer, row0)


def attention(dtype, q_rot, k_layer, v_layer, ctx_len):
    """Definition of the query-prefill attention; returns fp64 [n_q][Hq][d]."""
    q_rot = _chk(q_rot, "f32")
    n_q, n_q_heads, d = q_rot.shape
    n_kv, t_cap, _ = k_layer.shape
    assert k_layer.flags.c_contiguous and v_layer.flags.c_contiguous
    assert k_layer.dtype == _NP[dtype] and v_layer.dtype == _NP[dtype]
    assert ctx_len + n_q <= t_cap and n_q_heads % n_kv == 0
    out = np.empty((n_q, n_q_heads, d), np.float64)
    lib().kvo_attention(_DT[dtype], n_q_heads, n_kv, d, n_q, int(ctx_len), _p(q_rot),
                        _p(k_layer), _p(v_layer), int(t_cap), _p(out))
    return out


def query_prefill(dtype, q, k_new, v_new, inv_f, ctx_len, k_layer, v_layer, prerotated=False):
    """One layer of the query side: rope + append, then attention."""
    q_rot = query_rope_append(dtype, q, k_new, v_new, inv_f, ctx_len, k_layer, v_layer, prerotated)
    return attention(dtype, q_rot, k_layer, v_layer, ctx_len)
