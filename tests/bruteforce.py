"""float64 brute force of the serving path, written differently from the oracle:
explicit d x d block rotation matrices, an explicit [n_q][T+n_q] score matrix
with an explicit boolean mask.  Used only to pin the oracle on tiny inputs."""
import math

import numpy as np


def bf16_bits_to_f64(a):
    a = np.asarray(a, np.uint16)
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def widen(a, dtype):
    return bf16_bits_to_f64(a) if dtype == "bf16" else np.asarray(a, np.float64)


def rot_matrix(pos, inv_freq):
    """R_{Theta,pos}: element i pairs with i + d/2 (Eq. 1)."""
    h = len(inv_freq)
    d = 2 * h
    R = np.zeros((d, d))
    for i in range(h):
        a = float(pos) * float(inv_freq[i])
        c, s = math.cos(a), math.sin(a)
        R[i, i] = c
        R[i, i + h] = -s
        R[i + h, i] = s
        R[i + h, i + h] = c
    return R


def assemble(dtype, pk_k, pk_v, inv_freq, base_pos=0):
    """Exact (unrounded) realigned concatenation: K,V [layers][Hkv][base_pos+T][d] float64.
    Rows below base_pos are zero."""
    n_layers, n_kv, _, d = pk_k[0].shape
    T = base_pos + sum(p.shape[2] for p in pk_k)
    K = np.zeros((n_layers, n_kv, T, d))
    V = np.zeros((n_layers, n_kv, T, d))
    delta = base_pos
    for pk, pv in zip(pk_k, pk_v):
        n = pk.shape[2]
        R = rot_matrix(delta, inv_freq)
        K[:, :, delta:delta + n, :] = np.einsum("ef,lhtf->lhte", R, widen(pk, dtype))
        V[:, :, delta:delta + n, :] = widen(pv, dtype)
        delta += n
    return K, V


def attention(q_rot, K, V, ctx_len):
    """q_rot [n_q][Hq][d], K/V [Hkv][>=ctx_len+n_q][d] float64 -> O [n_q][Hq][d]."""
    n_q, n_qh, d = q_rot.shape
    n_kv = K.shape[0]
    g = n_qh // n_kv
    S = ctx_len + n_q
    out = np.zeros((n_q, n_qh, d))
    mask = np.zeros((n_q, S), bool)
    for t in range(n_q):
        mask[t, : ctx_len + t + 1] = True
    for hq in range(n_qh):
        h = hq // g
        scores = q_rot[:, hq, :] @ K[h, :S, :].T / math.sqrt(d)
        scores = np.where(mask, scores, -np.inf)
        scores -= scores.max(axis=1, keepdims=True)
        p = np.exp(scores)
        p /= p.sum(axis=1, keepdims=True)
        out[:, hq, :] = p @ V[h, :S, :]
    return out
