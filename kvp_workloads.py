"""Seeded synthetic RAG-shaped workloads shared by the tests, the smoke check
and the benchmark.

This module only *draws inputs*: packet lengths, retrieval lists, and K/V/Q
values.  It holds none of the method's arithmetic (no RoPE, no gather, no
attention) and imports neither the HIP binding nor the oracle.

Values come from a counter-based generator built from torch integer ops, so
the same (seed, tensor, packet, index) gives the same bits on the CPU and on
the GPU: value = NORMAL_TABLE[mix64(key + index) & 0xFFFF] * scale, where
NORMAL_TABLE is a 65536-entry inverse-CDF table of N(0,1) computed once on
the CPU in float64.  For bf16 workloads the table is rounded to bf16 first and
scale is a power of two, so every value is exactly representable.
"""
from dataclasses import dataclass, field
import math

import numpy as np
import torch

_MASK64 = (1 << 64) - 1


def _s64(x):
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)
_GOLD = _s64(0x9E3779B97F4A7C15)


def _lsr(x, s):
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x):
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _mix64_int(x):
    x &= _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def stream_key(seed, tensor_id, packet=0):
    """Scalar key of one logical tensor (python int, signed 64-bit)."""
    k = _mix64_int(seed * 0x9E3779B97F4A7C15 + 1)
    k = _mix64_int(k ^ (tensor_id * 0xD1B54A32D192ED03 + 2))
    k = _mix64_int(k ^ (packet * 0x8CB92BA72F3D8DD7 + 3))
    return _s64(k)


_TABLES = {}


def normal_table(dtype, device="cpu"):
    """65536-entry N(0,1) inverse-CDF table in ``dtype`` on ``device``."""
    key = (dtype, str(device))
    if key not in _TABLES:
        if (dtype, "cpu") not in _TABLES:
            u = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
            t = torch.special.ndtri(u).to(torch.float32)
            _TABLES[(dtype, "cpu")] = t.to(dtype)
        _TABLES[key] = _TABLES[(dtype, "cpu")].to(device)
    return _TABLES[key]


TENSOR_K, TENSOR_V, TENSOR_Q, TENSOR_KNEW, TENSOR_VNEW, TENSOR_HEADER_K, TENSOR_HEADER_V = 1, 2, 3, 4, 5, 6, 7


def normal_tensor(shape, seed, tensor_id, packet=0, scale=1.0, dtype=torch.bfloat16,
                  device="cpu", chunk=1 << 26):
    """Tensor of ``shape`` with N(0,1)*scale entries, reproducible bit for bit
    on any device.  ``scale`` must be a power of two for bf16."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=dtype, device=device)
    table = normal_table(dtype, device)
    key = stream_key(seed, tensor_id, packet)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        h = _mix64(idx * _GOLD + key) & 0xFFFF
        out[lo:hi] = table[h] * scale
    return out.view(*shape)


# --------------------------------------------------------------------------
# Workload recipes (shapes, length mix, retrieval pattern)
# --------------------------------------------------------------------------
@dataclass
class Request:
    packet_ids: list          # retrieval order = concatenation order
    n_q: int
    base_pos: int = 0


@dataclass
class Workload:
    name: str
    dtype: str                # "f32" | "bf16"
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    n_header: int
    n_trailer: int
    seed: int
    kv_scale: float
    packet_lens: np.ndarray   # [n_packets] total rows = N_h + L + N_t
    requests: list = field(default_factory=list)
    paged: bool = False
    block_size: int = 16
    prune: tuple = None       # (lo, hi): every (packet, layer) loses a seeded fraction in [lo, hi] of its rows
    shared_header: bool = False  # the first n_header rows are the same in every packet (global adapters, Sec. 4.1)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    def ctx_len(self, r):
        rq = self.requests[r]
        return rq.base_pos + int(sum(int(self.packet_lens[p]) for p in rq.packet_ids))

    def kept_rows(self, pid, layer):
        """Sorted rows of packet ``pid`` that a pruning pass kept in ``layer`` (a different,
        unstructured subset per layer), or None when the workload is not pruned."""
        if self.prune is None:
            return None
        n = int(self.packet_lens[pid])
        rng = np.random.default_rng([self.seed, 7, int(pid), int(layer)])
        n_keep = n - int(round(n * rng.uniform(*self.prune)))
        return np.sort(rng.choice(n, size=n_keep, replace=False))

    def layer_rows(self, r, layer):
        """Rows of request ``r``'s context in ``layer`` of the composed cache (= ctx_len(r)
        unless the workload is pruned)."""
        if self.prune is None:
            return self.ctx_len(r)
        rq = self.requests[r]
        return rq.base_pos + int(sum(len(self.kept_rows(p, layer)) for p in rq.packet_ids))

    def kv_bytes_per_token_layer(self):
        return 2 * self.n_kv_heads * self.head_dim * self.elem_bytes

    # -- value draws ------------------------------------------------------
    def packet_kv(self, pid, device="cpu", layers=None):
        """(K, V) of packet ``pid``: [n_layers][Hkv][len][d]."""
        n_l = self.n_layers if layers is None else layers
        shape = (n_l, self.n_kv_heads, int(self.packet_lens[pid]), self.head_dim)
        k = normal_tensor(shape, self.seed, TENSOR_K, pid, self.kv_scale, self.torch_dtype, device)
        v = normal_tensor(shape, self.seed, TENSOR_V, pid, self.kv_scale, self.torch_dtype, device)
        if self.shared_header:
            n_h = min(self.n_header, shape[2])
            hk, hv = self.header_kv(device, n_l)
            k[:, :, :n_h], v[:, :, :n_h] = hk[:, :, :n_h], hv[:, :, :n_h]
        return k, v

    def header_kv(self, device="cpu", layers=None):
        """(K, V) of the header rows all packets share: [n_layers][Hkv][n_header][d]."""
        n_l = self.n_layers if layers is None else layers
        shape = (n_l, self.n_kv_heads, self.n_header, self.head_dim)
        k = normal_tensor(shape, self.seed, TENSOR_HEADER_K, 0, self.kv_scale, self.torch_dtype, device)
        v = normal_tensor(shape, self.seed, TENSOR_HEADER_V, 0, self.kv_scale, self.torch_dtype, device)
        return k, v

    def query(self, r, layer, device="cpu"):
        """(Q, K_new, V_new) of request ``r`` at ``layer``; un-rotated."""
        n_q = self.requests[r].n_q
        tag = r * 1024 + layer
        q = normal_tensor((n_q, self.n_q_heads, self.head_dim), self.seed, TENSOR_Q, tag, 1.0,
                          self.torch_dtype, device)
        kn = normal_tensor((n_q, self.n_kv_heads, self.head_dim), self.seed, TENSOR_KNEW, tag,
                           self.kv_scale, self.torch_dtype, device)
        vn = normal_tensor((n_q, self.n_kv_heads, self.head_dim), self.seed, TENSOR_VNEW, tag,
                           self.kv_scale, self.torch_dtype, device)
        return q, kn, vn


def _uniform_lens(rng, n, lo, hi, extra):
    return (rng.integers(lo, hi + 1, size=n) + extra).astype(np.int64)


def tiny_fp32(seed=1001):
    """Config 1: 1 layer, 4/2 heads, d=64, fp32, 8 packets of 4+64+4 rows, k=2, n_q=16."""
    rng = np.random.default_rng(seed)
    lens = np.full(8, 72, np.int64)
    ids = [int(x) for x in rng.integers(0, 8, size=2)]
    return Workload("tiny_fp32", "f32", 1, 4, 2, 64, 1.0e4, 4, 4, seed, 1.0, lens,
                    [Request(ids, 16)])


def llama_k5(seed=1002, n_layers=32, n_packets=256):
    """Config 2: Llama-3.1-8B shape, 256 packets, L~U[256,1024]+8+8, k=5, n_q=32."""
    rng = np.random.default_rng(seed)
    lens = _uniform_lens(rng, n_packets, 256, 1024, 16)
    ids = [int(x) for x in rng.choice(n_packets, size=5, replace=False)]
    return Workload("llama_k5", "bf16", n_layers, 32, 8, 128, 5.0e5, 8, 8, seed, 0.5, lens,
                    [Request(ids, 32)])


def qwen_k20(seed=1003, n_layers=28, n_packets=1024):
    """Config 3: Qwen2.5-7B shape, 1024 packets, L~U[128,512]+8+8, k=20, n_q=64."""
    rng = np.random.default_rng(seed)
    lens = _uniform_lens(rng, n_packets, 128, 512, 16)
    ids = [int(x) for x in rng.choice(n_packets, size=20, replace=False)]
    return Workload("qwen_k20", "bf16", n_layers, 28, 4, 128, 1.0e6, 8, 8, seed, 0.5, lens,
                    [Request(ids, 64)])


def llama_long_b8(seed=1004, n_layers=1, n_packets=4096, batch=8, k=32, n_q=128):
    """Config 4: Llama shape, packets of exactly 8+512+8 rows, batch 8, k=32, n_q=128."""
    rng = np.random.default_rng(seed)
    lens = np.full(n_packets, 528, np.int64)
    reqs = [Request([int(x) for x in rng.choice(n_packets, size=k, replace=False)], n_q)
            for _ in range(batch)]
    return Workload("llama_long_b8", "bf16", n_layers, 32, 8, 128, 5.0e5, 8, 8, seed, 0.5, lens,
                    reqs)


def serving_mix(seed=1005, n_layers=1, n_packets=16384, n_req=64, sigma=0.6):
    """Config 5: 64 requests, k~U{3..16}, L lognormal (median 384, cap 2048, min 16) + 8+8,
    n_q~U{16..256}, Zipf(1.1) popularity over a seeded rank->id permutation, paged (block 16)."""
    rng = np.random.default_rng(seed)
    doc = np.exp(rng.normal(math.log(384.0), sigma, size=n_packets))
    lens = (np.clip(np.rint(doc), 16, 2048) + 16).astype(np.int64)
    perm = rng.permutation(n_packets)
    w = 1.0 / np.arange(1, n_packets + 1, dtype=np.float64) ** 1.1
    w /= w.sum()
    reqs = []
    for _ in range(n_req):
        k = int(rng.integers(3, 17))
        ranks = rng.choice(n_packets, size=k, replace=False, p=w)
        reqs.append(Request([int(perm[x]) for x in ranks], int(rng.integers(16, 257))))
    return Workload("serving_mix", "bf16", n_layers, 32, 8, 128, 5.0e5, 8, 8, seed, 0.5, lens,
                    reqs, paged=True, block_size=16)


def llama_8k(seed=1008, n_layers=32, n_packets=64, n_q=32, name="llama_8k"):
    """Headline point: Llama shape, k=16 packets of 8+496+8 = 512 rows -> T=8192, n_q=32."""
    rng = np.random.default_rng(seed)
    lens = np.full(n_packets, 512, np.int64)
    ids = [int(x) for x in rng.choice(n_packets, size=16, replace=False)]
    return Workload(name, "bf16", n_layers, 32, 8, 128, 5.0e5, 8, 8, seed, 0.5, lens,
                    [Request(ids, n_q)])


def llama_8k_pruned(seed=1009, n_layers=32, n_packets=64, rates=(0.1, 0.5)):
    """The headline point with every packet pruned offline: each (packet, layer) keeps its own
    random subset of rows, 10 % to 50 % removed (the range of compression rates of Sec. 5.4)."""
    w = llama_8k(seed, n_layers, n_packets, name="llama_8k_pruned")
    w.prune = tuple(rates)
    return w


def llama_8k_decode(seed=1008, n_layers=32, n_packets=64):
    """One generated token over the headline point's composed cache (n_q = 1)."""
    return llama_8k(seed, n_layers, n_packets, n_q=1, name="llama_8k_decode")


def random_small(seed, dtype="f32", d=8, n_q_heads=4, n_kv_heads=2, n_layers=2, n_packets=5,
                 k=3, n_q=5, max_len=9, n_req=1, base_pos=0, rope_base=1.0e4):
    """Small ragged case for brute-force tests (lengths down to 1 row)."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, max_len + 1, size=n_packets).astype(np.int64)
    reqs = [Request([int(x) for x in rng.integers(0, n_packets, size=k)], n_q, base_pos)
            for _ in range(n_req)]
    return Workload("random_small", dtype, n_layers, n_q_heads, n_kv_heads, d, rope_base, 0, 0,
                    seed, 1.0 if dtype == "f32" else 0.5, lens, reqs)


def to_numpy(t):
    """torch tensor -> numpy in the oracle's convention (bf16 as uint16 bits)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
