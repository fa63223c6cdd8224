"""Pins of the CPU oracle against things other than itself: closed forms,
Eq. 1's algebra, brute force with explicit matrices, a library SDPA, and the
invariants the method fixes.  CPU only."""
import math

import numpy as np
import pytest
import torch

import kvp_workloads as W
import oracle
from tests import bruteforce as bf


def _np(t):
    return W.to_numpy(t)


def _packets(w, ids):
    ks, vs = [], []
    for p in ids:
        k, v = w.packet_kv(p)
        ks.append(_np(k))
        vs.append(_np(v))
    return ks, vs


# --------------------------------------------------------------------------
# RoPE pieces (Eq. 1)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("base,d", [(1.0e4, 64), (5.0e5, 128), (1.0e6, 128), (1.0e4, 2)])
def test_inv_freq_closed_form(base, d):
    f = oracle.inv_freq(base, d)
    assert f.dtype == np.float32 and f.shape == (d // 2,)
    assert f[0] == 1.0
    for i in range(d // 2):
        exact = base ** (-2.0 * i / d)
        assert abs(float(f[i]) - exact) <= 2.0 ** -24 * exact
    if d >= 4:
        assert abs(float(f[-1]) * base ** ((d - 2.0) / d) - 1.0) < 1e-6


@pytest.mark.parametrize("pos", [0, 1, 7, 144, 8191, 100000])
def test_rotation_equals_explicit_matrix(pos):
    rng = np.random.default_rng(pos + 1)
    d = 16
    f = oracle.inv_freq(1.0e4, d)
    x = rng.standard_normal(d).astype(np.float32)
    y = oracle.rotate(x, pos, f)
    ref = bf.rot_matrix(pos, f) @ x.astype(np.float64)
    assert np.max(np.abs(y - ref)) < 5e-7 * (1 + np.max(np.abs(x)))
    # a rotation preserves the norm of every pair
    h = d // 2
    assert np.allclose(y[:h] ** 2 + y[h:] ** 2, x[:h] ** 2 + x[h:] ** 2, rtol=1e-5)


def test_rotation_pairs_i_with_i_plus_half():
    # a unit vector on axis i moves only into axes i and i + d/2, by angle pos*theta_i
    d, pos = 8, 3
    f = oracle.inv_freq(1.0e4, d)
    for i in range(d // 2):
        e = np.zeros(d, np.float32)
        e[i] = 1.0
        y = oracle.rotate(e, pos, f)
        a = pos * float(f[i])
        want = np.zeros(d)
        want[i], want[i + d // 2] = math.cos(a), math.sin(a)
        assert np.max(np.abs(y - want)) < 1e-6


@pytest.mark.parametrize("S,delta", [(0, 5), (17, 100), (300, -300), (300, -7), (12, 0), (0, 0)])
def test_rotation_composition(S, delta):
    # Eq. 1: R_Delta R_S = R_{S+Delta} for every integer Delta, negative included
    d = 64
    f = oracle.inv_freq(1.0e4, d)
    x = np.random.default_rng(5).standard_normal(d).astype(np.float32)
    two_step = oracle.rotate(oracle.rotate(x, S, f), delta, f)
    one_step = oracle.rotate(x, S + delta, f)
    assert np.max(np.abs(two_step - one_step)) < 2e-5


def test_relative_position_property():
    # <R_m q, R_n k> depends on m - n only
    d = 64
    f = oracle.inv_freq(5.0e5, d)
    rng = np.random.default_rng(9)
    q = rng.standard_normal(d).astype(np.float32)
    k = rng.standard_normal(d).astype(np.float32)
    base = float(np.dot(oracle.rotate(q, 40, f).astype(np.float64), oracle.rotate(k, 13, f)))
    for shift in (1, 100, 5000, -13):
        s = float(np.dot(oracle.rotate(q, 40 + shift, f).astype(np.float64),
                         oracle.rotate(k, 13 + shift, f)))
        assert abs(s - base) < 2e-4
    other = float(np.dot(oracle.rotate(q, 41, f).astype(np.float64), oracle.rotate(k, 13, f)))
    assert abs(other - base) > 1e-3  # and it does depend on m - n


def test_rotation_zero_is_value_identity():
    d = 32
    f = oracle.inv_freq(1.0e4, d)
    x = np.random.default_rng(2).standard_normal(d).astype(np.float32)
    assert np.array_equal(oracle.rotate(x, 0, f), x)


# --------------------------------------------------------------------------
# bf16 rounding and the "separately rounded fp32" reading
# --------------------------------------------------------------------------
def test_bf16_assemble_matches_torch_rounding_bit_for_bit():
    w = W.random_small(21, dtype="bf16", d=16, n_layers=1, n_packets=3, k=3, max_len=40)
    ids = w.requests[0].packet_ids
    ks, vs = _packets(w, ids)
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    K, V, ctx = oracle.assemble("bf16", ks, vs, f)
    h = w.head_dim // 2
    delta = 0
    for j, p in enumerate(ids):
        kt, vt = w.packet_kv(p)
        n = kt.shape[2]
        c = torch.tensor([np.float32(math.cos(float(delta) * float(fi))) for fi in f])
        s = torch.tensor([np.float32(math.sin(float(delta) * float(fi))) for fi in f])
        x, y = kt[..., :h].float(), kt[..., h:].float()
        lo = (x * c) - (y * s)          # torch CPU: each op rounded to fp32, no fusion
        hi = (y * c) + (x * s)
        want = torch.cat([lo, hi], -1).to(torch.bfloat16)   # round to nearest even
        assert np.array_equal(_np(want), K[:, :, delta:delta + n, :])
        assert np.array_equal(_np(vt), V[:, :, delta:delta + n, :])
        delta += n
    assert ctx == delta


def _angle_with_cos(target):
    """An fp32 angle a with (float)cos((double)a) == target exactly."""
    a = np.float32(math.acos(float(target)))
    for _ in range(2000):
        if np.float32(math.cos(float(a))) == np.float32(target):
            return a
        a = np.nextafter(a, np.float32(0 if np.float32(math.cos(float(a))) < target else 4))
    raise AssertionError("no such angle")


@pytest.mark.parametrize("cos_val,bits", [
    (1.0 - 3 * 2.0 ** -9, 0x3F7E),   # halfway between 0x3F7E (even) and 0x3F7F: goes down
    (1.0 - 1 * 2.0 ** -9, 0x3F80),   # halfway between 0x3F7F and 0x3F80 (even): goes up
    (1.0 - 5 * 2.0 ** -10, 0x3F7F),   # above the midpoint of 0x3F7E..0x3F7F: nearest
])
def test_bf16_ties_round_to_even(cos_val, bits):
    # K = (1, 0) rotated by an angle whose fp32 cosine is exactly cos_val gives lo = cos_val,
    # which the bf16 store must round to nearest, ties to even.
    a = _angle_with_cos(cos_val)
    f = np.array([a], np.float32)
    one = np.array([0x3F80, 0x0000], np.uint16).reshape(1, 1, 1, 2)
    K, V, ctx = oracle.assemble("bf16", [one, one], [one, one], f)   # 2nd packet sits at Delta=1
    assert ctx == 2
    assert K[0, 0, 0, 0] == 0x3F80 and K[0, 0, 0, 1] == 0
    assert K[0, 0, 1, 0] == bits
    # sign symmetry
    neg = np.array([0xBF80, 0x0000], np.uint16).reshape(1, 1, 1, 2)
    K, _, _ = oracle.assemble("bf16", [one, neg], [one, neg], f)
    assert K[0, 0, 1, 0] == bits | 0x8000


def test_denormals_are_kept():
    """Subnormal inputs and results go through the rotation unflushed (closed forms in exact
    powers of two, and numpy's separately rounded fp32 scalar ops on random subnormals)."""
    from fractions import Fraction

    def to_grid(fr, ulp_exp):
        """Nearest multiple of 2^ulp_exp, ties to even, as (multiple, exact?)."""
        q = fr / Fraction(2) ** ulp_exp
        n = q.numerator // q.denominator
        rem = q - n
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2):
            n += 1
        return n

    a = np.float32(0.7)
    f = np.array([a], np.float32)
    c1, s1 = np.float32(math.cos(float(a))), np.float32(math.sin(float(a)))
    # fp32: K = (2^-140, 0) at Delta = 1 -> lo = fl(2^-140 cos), hi = fl(2^-140 sin): both subnormal,
    # multiples of 2^-149 found by exact rational arithmetic
    x = np.float32(2.0 ** -140)
    pk = np.array([x, 0], np.float32).reshape(1, 1, 1, 2)
    K, V, _ = oracle.assemble("f32", [pk, pk], [pk, pk], f)
    assert K[0, 0, 0].view(np.uint32).tolist() == [0x00000200, 0]          # Delta = 0: the value itself, 2^-140
    want_lo = to_grid(Fraction(float(c1)) * Fraction(2) ** -140, -149)
    want_hi = to_grid(Fraction(float(s1)) * Fraction(2) ** -140, -149)
    assert 0 < want_lo < 0x00800000 and 0 < want_hi < 0x00800000            # subnormal bit patterns are the multiples
    assert int(K[0, 0, 1, 0].view(np.uint32)) == want_lo
    assert int(K[0, 0, 1, 1].view(np.uint32)) == want_hi
    assert V[0, 0, 1].view(np.uint32).tolist() == [0x00000200, 0]
    # bf16: the subnormal 0x0040 (2^-127) times cos, sin lands on bf16's subnormal grid 2^-133
    pb = np.array([0x0040, 0x0000], np.uint16).reshape(1, 1, 1, 2)
    K, V, _ = oracle.assemble("bf16", [pb, pb], [pb, pb], f)
    assert K[0, 0, 0].tolist() == [0x0040, 0]
    # (the fp32 products 2^-127 cos and 2^-127 sin are exact multiples of 2^-150?  no: fp32 rounds
    # them to 2^-149 first, then the store rounds to 2^-133; both steps ties-to-even)
    def two_step(cf):
        n32 = to_grid(Fraction(float(cf)) * Fraction(2) ** -127, -149)
        return to_grid(Fraction(n32) * Fraction(2) ** -149, -133)
    assert int(K[0, 0, 1, 0]) == two_step(c1) and int(K[0, 0, 1, 1]) == two_step(s1)
    assert 0 < int(K[0, 0, 1, 0]) < 0x0080
    # random subnormal and tiny normal keys against numpy scalar arithmetic (each op rounded to fp32)
    rng = np.random.default_rng(5)
    d = 8
    fr = oracle.inv_freq(1.0e4, d)
    bits = rng.integers(1, 0x01000000, size=(1, 1, 6, d)).astype(np.uint32)   # up to 2^-125, mostly subnormal
    bits ^= (rng.integers(0, 2, size=bits.shape).astype(np.uint32) << 31)
    kk = bits.view(np.float32)
    K, _, _ = oracle.assemble("f32", [kk[:, :, :2], kk[:, :, 2:]], [kk[:, :, :2], kk[:, :, 2:]], fr)
    h = d // 2
    for t in range(2, 6):                           # the second packet sits at Delta = 2
        for i in range(h):
            ang = 2.0 * float(fr[i])
            c, sn = np.float32(math.cos(ang)), np.float32(math.sin(ang))
            xv, yv = kk[0, 0, t, i], kk[0, 0, t, i + h]
            lo = np.float32(np.float32(xv * c) - np.float32(yv * sn))
            hi = np.float32(np.float32(yv * c) + np.float32(xv * sn))
            assert K[0, 0, t, i].view(np.uint32) == lo.view(np.uint32)
            assert K[0, 0, t, i + h].view(np.uint32) == hi.view(np.uint32)
    assert np.count_nonzero(K[0, 0, 2:]) == 4 * d   # nothing was flushed to zero


# --------------------------------------------------------------------------
# Brute force on tiny inputs (explicit matrices, explicit mask, float64)
# --------------------------------------------------------------------------
def _end_to_end(w, r=0, prerotated=False):
    rq = w.requests[r]
    ks, vs = _packets(w, rq.packet_ids)
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    n_q = rq.n_q
    ctx_expected = w.ctx_len(r)
    t_cap = ctx_expected + n_q + 3
    shape = (w.n_layers, w.n_kv_heads, t_cap, w.head_dim)
    npdt = np.float32 if w.dtype == "f32" else np.uint16
    K = np.zeros(shape, npdt)
    V = np.zeros(shape, npdt)
    K, V, ctx = oracle.assemble(w.dtype, ks, vs, f, rq.base_pos, t_cap, K, V)
    assert ctx == ctx_expected
    outs = []
    for layer in range(w.n_layers):
        q, kn, vn = w.query(r, layer)
        o = oracle.query_prefill(w.dtype, _np(q), _np(kn), _np(vn), f, ctx, K[layer], V[layer],
                                 prerotated)
        outs.append(o)
    return ks, vs, f, K, V, ctx, outs


CASES = [
    dict(seed=1, d=2, n_q_heads=1, n_kv_heads=1, k=1, n_q=1, max_len=1),
    dict(seed=2, d=4, n_q_heads=2, n_kv_heads=2, k=3, n_q=4),
    dict(seed=3, d=8, n_q_heads=7, n_kv_heads=1, k=3, n_q=5),
    dict(seed=4, d=8, n_q_heads=4, n_kv_heads=2, k=0, n_q=6),
    dict(seed=5, d=8, n_q_heads=4, n_kv_heads=2, k=3, n_q=3, base_pos=11),
    dict(seed=6, d=16, n_q_heads=14, n_kv_heads=2, k=4, n_q=9, max_len=30),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CASES, ids=[str(c["seed"]) for c in CASES])
def test_brute_force_tiny(case, dtype):
    w = W.random_small(dtype=dtype, **case)
    ks, vs, f, K, V, ctx, outs = _end_to_end(w)
    rq = w.requests[0]
    n_q = rq.n_q
    if ks:
        Kx, Vx = bf.assemble(dtype, ks, vs, f, rq.base_pos)
        Ko = bf.widen(K[:, :, :ctx], dtype)
        rel = 2.0 ** -8 if dtype == "bf16" else 1e-6
        sel = slice(rq.base_pos, ctx)
        assert np.all(np.abs(Ko[:, :, sel] - Kx[:, :, sel]) <= rel * np.abs(Kx[:, :, sel]) + 1e-6)
        assert np.array_equal(bf.widen(V[:, :, sel], dtype), Vx[:, :, sel])
    for layer in range(w.n_layers):
        q, kn, vn = w.query(0, layer)
        qn, knn, vnn = (bf.widen(_np(x), dtype) for x in (q, kn, vn))
        # query side by explicit matrices, float64
        q_rot = np.stack([np.einsum("ef,hf->he", bf.rot_matrix(ctx + t, f), qn[t])
                          for t in range(n_q)])
        Kl = bf.widen(K[layer], dtype).copy()
        Vl = bf.widen(V[layer], dtype).copy()
        for t in range(n_q):
            want = np.einsum("ef,hf->he", bf.rot_matrix(ctx + t, f), knn[t])
            got = Kl[:, ctx + t, :]
            rel = 2.0 ** -8 if dtype == "bf16" else 1e-6
            assert np.all(np.abs(got - want) <= rel * np.abs(want) + 1e-6)
            assert np.array_equal(Vl[:, ctx + t, :], vnn[t])
        # rows below base_pos are the caller's: the oracle leaves the zeros we put there
        assert not Kl[:, :rq.base_pos].any()
        ref = bf.attention(q_rot, Kl, Vl, ctx)
        assert np.max(np.abs(outs[layer] - ref)) < 2e-5


def test_brute_force_config1():
    w = W.tiny_fp32()
    assert (w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim) == (1, 4, 2, 64)
    assert w.ctx_len(0) == 144 and w.requests[0].n_q == 16
    ks, vs, f, K, V, ctx, outs = _end_to_end(w)
    Kx, Vx = bf.assemble("f32", ks, vs, f)
    assert np.max(np.abs(K[:, :, :ctx] - Kx)) < 2e-5
    assert np.array_equal(V[:, :, :ctx].astype(np.float64), Vx)
    q, kn, vn = w.query(0, 0)
    q_rot = np.stack([np.einsum("ef,hf->he", bf.rot_matrix(ctx + t, f), _np(q)[t].astype(float))
                      for t in range(16)])
    ref = bf.attention(q_rot, K[0].astype(np.float64), V[0].astype(np.float64), ctx)
    assert np.max(np.abs(outs[0] - ref)) < 2e-5


# --------------------------------------------------------------------------
# One packet, no adapters  ==  plain causal attention (library SDPA)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("g", [1, 4])
def test_one_packet_reduces_to_plain_causal_attention(g):
    torch.manual_seed(0)
    L, n_q, n_kv, d = 37, 6, 2, 32
    n_qh = g * n_kv
    base = 1.0e4
    S = L + n_q
    k_raw = torch.randn(S, n_kv, d)
    v_raw = torch.randn(S, n_kv, d)
    q_raw = torch.randn(S, n_qh, d)

    # textbook route, all in torch: rotate everything at positions 0..S-1, causal SDPA
    inv = torch.tensor([base ** (-2.0 * i / d) for i in range(d // 2)], dtype=torch.float64)
    ang = torch.arange(S, dtype=torch.float64)[:, None] * inv[None, :]
    cos, sin = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

    def rope(x):
        x = x.double()
        a, b = x[..., : d // 2], x[..., d // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], -1)

    qr, kr = rope(q_raw), rope(k_raw)
    kk = kr.permute(1, 0, 2).repeat_interleave(g, 0)          # [Hq][S][d], head hq -> kv hq//g
    vv = v_raw.double().permute(1, 0, 2).repeat_interleave(g, 0)
    ref = torch.nn.functional.scaled_dot_product_attention(
        qr.permute(1, 0, 2)[None], kk[None], vv[None], is_causal=True)[0]
    ref = ref.permute(1, 0, 2)[L:].numpy()                    # last n_q rows

    # packet route: the packet holds the first L rows, keys already rotated at 0..L-1
    pk = kr[:L].float().permute(1, 0, 2)[None].contiguous().numpy()     # [1][Hkv][L][d]
    pv = v_raw[:L].permute(1, 0, 2)[None].contiguous().numpy()
    f = oracle.inv_freq(base, d)
    K, V, ctx = oracle.assemble("f32", [pk], [pv], f, 0, S)
    assert ctx == L
    out = oracle.query_prefill("f32", q_raw[L:].numpy(), k_raw[L:].numpy(), v_raw[L:].numpy(),
                               f, ctx, K[0], V[0])
    assert np.max(np.abs(out - ref)) < 1e-5


# --------------------------------------------------------------------------
# Concatenation == K/V laid out by hand
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_concatenation_equals_hand_laid_cache(dtype):
    w = W.random_small(31, dtype=dtype, d=8, k=4, n_packets=6, max_len=12, n_q=4)
    ks, vs, f, K, V, ctx, outs = _end_to_end(w)
    ids = w.requests[0].packet_ids
    npdt = np.float32 if dtype == "f32" else np.uint16
    t_cap = K.shape[2]
    Kh = np.zeros_like(K)
    Vh = np.zeros_like(V)
    h = w.head_dim // 2
    row = 0
    for j, p in enumerate(ids):
        kt, vt = w.packet_kv(p)
        n = kt.shape[2]
        c = np.array([np.float32(math.cos(float(row) * float(x))) for x in f], np.float32)
        s = np.array([np.float32(math.sin(float(row) * float(x))) for x in f], np.float32)
        x = kt[..., :h].float().numpy()
        y = kt[..., h:].float().numpy()
        lo = (x * c).astype(np.float32) - (y * s).astype(np.float32)
        hi = (y * c).astype(np.float32) + (x * s).astype(np.float32)
        rot = torch.from_numpy(np.concatenate([lo, hi], -1)).to(w.torch_dtype)
        Kh[:, :, row:row + n] = _np(rot)
        Vh[:, :, row:row + n] = _np(vt)
        row += n
    assert row == ctx
    assert np.array_equal(Kh[:, :, :ctx], K[:, :, :ctx])
    assert np.array_equal(Vh[:, :, :ctx], V[:, :, :ctx])
    # attending over the hand-laid cache gives the same bits as the assembled route
    for layer in range(w.n_layers):
        q, kn, vn = w.query(0, layer)
        o = oracle.query_prefill(dtype, _np(q), _np(kn), _np(vn), f, ctx, Kh[layer], Vh[layer])
        assert np.array_equal(o, outs[layer])
    assert npdt == K.dtype and t_cap >= ctx


# --------------------------------------------------------------------------
# Packet order permutes only what the method defines
# --------------------------------------------------------------------------
def test_packet_order_permutes_blocks():
    w = W.random_small(41, dtype="f32", d=8, k=4, n_packets=4, max_len=10, n_layers=1)
    ids = [0, 1, 2, 3]
    perm = [2, 0, 3, 1]
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    lens = [int(w.packet_lens[p]) for p in range(4)]

    def run(order):
        ks, vs = _packets(w, order)
        K, V, ctx = oracle.assemble("f32", ks, vs, f)
        starts, row = {}, 0
        for p in order:
            starts[p] = row
            row += lens[p]
        return K, V, starts

    K1, V1, s1 = run(ids)
    K2, V2, s2 = run(perm)
    for p in ids:
        n = lens[p]
        # V blocks merely move
        assert np.array_equal(V1[:, :, s1[p]:s1[p] + n], V2[:, :, s2[p]:s2[p] + n])
        # K block in the second order = R_{s2 - s1} applied to the block in the first order
        blk = K1[0, :, s1[p]:s1[p] + n].astype(np.float64)
        want = np.einsum("ef,htf->hte", bf.rot_matrix(s2[p] - s1[p], f), blk)
        assert np.max(np.abs(K2[0, :, s2[p]:s2[p] + n] - want)) < 2e-5


def test_order_invariance_without_rope():
    # with theta = 0 (no positional signal) attention over a set of packets ignores their order
    w = W.random_small(43, dtype="f32", d=8, k=3, n_packets=3, max_len=10, n_layers=1, n_q=4)
    f = np.zeros(w.head_dim // 2, np.float32)
    q, kn, vn = (_np(x) for x in w.query(0, 0))
    outs = []
    for order in ([0, 1, 2], [2, 1, 0], [1, 2, 0]):
        ks, vs = _packets(w, order)
        ctx = sum(k.shape[2] for k in ks)
        K, V, c2 = oracle.assemble("f32", ks, vs, f, 0, ctx + 4)
        outs.append(oracle.query_prefill("f32", q, kn, vn, f, ctx, K[0], V[0]))
    assert np.max(np.abs(outs[0] - outs[1])) < 1e-9
    assert np.max(np.abs(outs[0] - outs[2])) < 1e-9


# --------------------------------------------------------------------------
# Softmax invariants
# --------------------------------------------------------------------------
def test_attention_is_a_convex_combination_of_values():
    w = W.random_small(51, dtype="f32", d=8, k=3, n_q=5, n_layers=1)
    ks, vs, f, K, V, ctx, outs = _end_to_end(w)
    o = outs[0]
    g = w.n_q_heads // w.n_kv_heads
    for t in range(w.requests[0].n_q):
        for hq in range(w.n_q_heads):
            vis = V[0, hq // g, : ctx + t + 1].astype(np.float64)
            assert np.all(o[t, hq] <= vis.max(0) + 1e-12)
            assert np.all(o[t, hq] >= vis.min(0) - 1e-12)


def test_constant_values_come_back_unchanged_and_first_row_sees_prefix_plus_itself():
    d, n_kv, n_qh = 8, 1, 2
    f = oracle.inv_freq(1.0e4, d)
    rng = np.random.default_rng(3)
    pk = rng.standard_normal((1, n_kv, 5, d)).astype(np.float32)
    pv = np.broadcast_to(np.arange(d, dtype=np.float32), (1, n_kv, 5, d)).copy()
    K, V, ctx = oracle.assemble("f32", [pk], [pv], f, 0, 8)
    q = rng.standard_normal((3, n_qh, d)).astype(np.float32)
    kn = rng.standard_normal((3, n_kv, d)).astype(np.float32)
    vn = np.broadcast_to(np.arange(d, dtype=np.float32), (3, n_kv, d)).copy()
    o = oracle.query_prefill("f32", q, kn, vn, f, ctx, K[0], V[0])
    assert np.max(np.abs(o - np.arange(d))) < 1e-12
    # k = 0, one query token: it sees only itself, so O = V_new exactly
    K0 = np.zeros((n_kv, 4, d), np.float32)
    V0 = np.zeros((n_kv, 4, d), np.float32)
    vn1 = rng.standard_normal((1, n_kv, d)).astype(np.float32)
    o1 = oracle.query_prefill("f32", q[:1], kn[:1], vn1, f, 0, K0, V0)
    assert np.array_equal(o1[0, 0], vn1[0, 0].astype(np.float64))
    assert np.array_equal(o1[0, 1], vn1[0, 0].astype(np.float64))


def test_causal_mask_among_query_tokens():
    # changing a later query token's K/V must not change an earlier token's output
    w = W.random_small(61, dtype="f32", d=8, k=2, n_q=4, n_layers=1)
    ks, vs, f, K, V, ctx, outs = _end_to_end(w)
    q, kn, vn = (_np(x).copy() for x in w.query(0, 0))
    kn[3] += 5.0
    vn[3] -= 7.0
    K2, V2 = K[0].copy(), V[0].copy()
    o2 = oracle.query_prefill("f32", q, kn, vn, f, ctx, K2, V2)
    assert np.array_equal(o2[:3], outs[0][:3])
    assert not np.array_equal(o2[3], outs[0][3])


def test_prerotated_flag_skips_the_rotation():
    w = W.random_small(71, dtype="f32", d=8, k=2, n_q=3, n_layers=1)
    ks, vs, f, K, V, ctx, outs = _end_to_end(w)
    q, kn, vn = (_np(x) for x in w.query(0, 0))
    q_r = np.stack([[oracle.rotate(q[t, h], ctx + t, f) for h in range(q.shape[1])]
                    for t in range(3)]).astype(np.float32)
    k_r = np.stack([[oracle.rotate(kn[t, h], ctx + t, f) for h in range(kn.shape[1])]
                    for t in range(3)]).astype(np.float32)
    K2, V2 = K[0].copy(), V[0].copy()
    o = oracle.query_prefill("f32", q_r, k_r, vn, f, ctx, K2, V2, prerotated=True)
    assert np.array_equal(o, outs[0])
    assert np.array_equal(K2, K[0])


# --------------------------------------------------------------------------
# Delta = 0 and the closed-form flop count
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_first_packet_at_position_zero_is_a_value_copy(dtype):
    w = W.random_small(81, dtype=dtype, d=8, k=2, max_len=12)
    ids = w.requests[0].packet_ids
    ks, vs = _packets(w, ids)
    f = oracle.inv_freq(w.rope_base, w.head_dim)
    K, V, ctx = oracle.assemble(dtype, ks, vs, f)
    n = ks[0].shape[2]
    assert np.array_equal(bf.widen(K[:, :, :n], dtype), bf.widen(ks[0], dtype))
    assert np.array_equal(V[:, :, :n], vs[0])


def test_rotating_keys_only_is_consistent_with_the_papers_printed_flop_range():
    # Not a pin of any oracle function: a check of the reading that only the keys are rotated.
    # Sec. 5.2: KV Packet's pre-generation FLOPs are the RoPE realignment alone, and Sec. 5.3
    # prints them as 6.50e-6 .. 1.04e-5 of a full recompute.  Only K is rotated: 4 mul + 2 add
    # per (i, i+d/2) pair -> 3 flop per K element.
    lines = [l.split() for l in open(__file__.replace("test_oracle_pins.py",
                                                      "golden/paper_flops_range.txt"))
             if l.strip() and not l.startswith("#")]
    lo, hi = float(lines[0][0]), float(lines[0][1])
    n_layers, n_kv, d = 32, 8, 128
    realign = 3 * n_kv * d * n_layers                     # flop per context token
    assert realign == 98304
    params = 8.03e9 - 128256 * 4096                       # Llama-3.1-8B without the input embedding
    full = 2 * params                                     # forward flop per token, attention excluded
    frac = realign / full
    assert lo <= frac <= hi


# --------------------------------------------------------------------------
# Compressed packets (Sec. 5.4): per layer a packet keeps a subset of its rows
# --------------------------------------------------------------------------
def _pruned_case(dtype, seed=21, d=8, n_kv=2, lens=(9, 1, 14), keep_prob=0.6):
    """Packets of one layer + the rows each keeps (sorted, possibly none)."""
    rng = np.random.default_rng(seed)
    w = W.random_small(seed, dtype=dtype, d=d, n_q_heads=2 * n_kv, n_kv_heads=n_kv, n_layers=1,
                       n_packets=len(lens), k=len(lens), n_q=4)
    f = oracle.inv_freq(w.rope_base, d)
    ks, vs, keeps = [], [], []
    for j, L in enumerate(lens):
        k = W.normal_tensor((1, n_kv, L, d), seed, 1, j, 1.0, w.torch_dtype)
        v = W.normal_tensor((1, n_kv, L, d), seed, 2, j, 1.0, w.torch_dtype)
        ks.append(_np(k)), vs.append(_np(v))
        keep = np.flatnonzero(rng.random(L) < keep_prob)
        keeps.append(keep)
    keeps[1] = np.array([0])            # a one-row packet keeps its row
    return w, f, ks, vs, keeps


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("base_pos", [0, 5])
def test_pruning_commutes_with_realignment(dtype, base_pos):
    """Realigning the kept rows of compressed packets (spans = the uncompressed lengths) gives,
    bit for bit, the rows a full assembly puts at those places: Eq. 1 rotates every key of a
    packet by the same Delta_j whatever its own position.  The full assembly is the function the
    pins above fix; the selection is plain indexing."""
    w, f, ks, vs, keeps = _pruned_case(dtype)
    lens = [k.shape[2] for k in ks]
    K, V, ctx = oracle.assemble(dtype, ks, vs, f, base_pos)
    pk = [np.ascontiguousarray(k[0][:, keep]) for k, keep in zip(ks, keeps)]
    pv = [np.ascontiguousarray(v[0][:, keep]) for v, keep in zip(vs, keeps)]
    Kc, Vc, rows, pos_end = oracle.assemble_layer_spans(dtype, pk, pv, lens, f, base_pos)
    assert rows == sum(len(k) for k in keeps) and pos_end == ctx == base_pos + sum(lens)
    sel = np.concatenate([base_pos + sum(lens[:j]) + keep for j, keep in enumerate(keeps)])
    assert np.array_equal(Kc, K[0][:, sel]) and np.array_equal(Vc, V[0][:, sel])


def test_uncompressed_spans_reduce_to_plain_assembly():
    w, f, ks, vs, _ = _pruned_case("bf16")
    lens = [k.shape[2] for k in ks]
    K, V, ctx = oracle.assemble("bf16", ks, vs, f, 3, t_cap=3 + sum(lens))
    Kc, Vc, rows, pos_end = oracle.assemble_layer_spans("bf16", [k[0] for k in ks], [v[0] for v in vs], lens, f, 3)
    assert rows == sum(lens) and pos_end == ctx
    assert np.array_equal(Kc, K[0][:, 3:]) and np.array_equal(Vc, V[0][:, 3:])


def test_pruned_attention_against_brute_force_with_explicit_positions():
    """Float64 brute force from the un-rotated keys: kept row s of packet j sits at position
    Delta_j + s with Delta_j counted in uncompressed lengths, the query at the sum of the
    lengths + t; an explicit score matrix over the kept rows and the query rows."""
    dtype = "f32"
    w, f, ks_raw, vs, keeps = _pruned_case(dtype, seed=33, lens=(6, 11, 1, 8))
    lens = [k.shape[2] for k in ks_raw]
    d, n_kv = w.head_dim, w.n_kv_heads
    # what a packet stores: its keys rotated at their local positions 0 .. len-1
    stored = []
    for k in ks_raw:
        st = np.stack([[oracle.rotate(k[0][h, s], s, f) for s in range(k.shape[2])] for h in range(n_kv)])
        stored.append(st.astype(np.float32))
    pk = [np.ascontiguousarray(st[:, keep]) for st, keep in zip(stored, keeps)]
    pv = [np.ascontiguousarray(v[0][:, keep]) for v, keep in zip(vs, keeps)]
    base_pos = 2
    n_q = w.requests[0].n_q
    rows_total = sum(len(k) for k in keeps)
    Kc, Vc, rows, pos_end = oracle.assemble_layer_spans(dtype, pk, pv, lens, f, base_pos, t_cap=rows_total + n_q)
    q, kn, vn = (_np(x) for x in w.query(0, 0))
    out = oracle.query_prefill_at(dtype, q, kn, vn, f, rows, pos_end, Kc, Vc)
    # brute force
    Kb = np.zeros((n_kv, rows_total + n_q, d)); Vb = np.zeros_like(Kb)
    at = 0
    for j, keep in enumerate(keeps):
        delta = base_pos + sum(lens[:j])
        for s in keep:
            R = bf.rot_matrix(delta + int(s), f)
            Kb[:, at] = np.einsum("ef,hf->he", R, ks_raw[j][0][:, s].astype(np.float64))
            Vb[:, at] = vs[j][0][:, s]
            at += 1
    pos_q = base_pos + sum(lens)
    assert at == rows and pos_end == pos_q
    q_rot = np.stack([np.einsum("ef,hf->he", bf.rot_matrix(pos_q + t, f), q[t].astype(np.float64)) for t in range(n_q)])
    for t in range(n_q):
        Kb[:, at + t] = np.einsum("ef,hf->he", bf.rot_matrix(pos_q + t, f), kn[t].astype(np.float64))
        Vb[:, at + t] = vn[t]
    ref = bf.attention(q_rot, Kb, Vb, rows)
    assert np.max(np.abs(out - ref)) < 3e-5
    # the appended rows sit behind the kept rows, at the query's positions
    assert np.max(np.abs(Kc[:, rows:rows + n_q].astype(np.float64) - Kb[:, rows:])) < 3e-5
    assert np.array_equal(Vc[:, rows:rows + n_q].astype(np.float64), Vb[:, rows:])
