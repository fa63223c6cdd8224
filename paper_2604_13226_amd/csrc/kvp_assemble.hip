// kvp_assemble.hip -- K1: gather the retrieved packets into the per-layer cache and
// realign their keys (Sec. 3.1, Eq. 1; Sec. 4.2.1 step 4).
//
// HBM-bound: every K and V element of the context is read once and written once; the
// rotation is 3 flop per K element.  The rotation angle Delta_j * theta_i does not depend
// on the row inside a packet, so each thread keeps the cos/sin of its column chunk in
// registers for the whole tile and only streams 16-byte K/V vectors through.
#include "kvp_device.h"

#pragma clang fp contract(off)  // products and sums are rounded separately, as the oracle's

namespace kvp {

template <typename T> struct Vec16;
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16_t> { static constexpr int N = 8; };

__device__ __forceinline__ void unpack(const uint4 &u, float (&x)[4])
{
    x[0] = __uint_as_float(u.x); x[1] = __uint_as_float(u.y);
    x[2] = __uint_as_float(u.z); x[3] = __uint_as_float(u.w);
}
__device__ __forceinline__ void unpack(const uint4 &u, float (&x)[8])
{
    x[0] = __uint_as_float(u.x << 16); x[1] = __uint_as_float(u.x & 0xFFFF0000u);
    x[2] = __uint_as_float(u.y << 16); x[3] = __uint_as_float(u.y & 0xFFFF0000u);
    x[4] = __uint_as_float(u.z << 16); x[5] = __uint_as_float(u.z & 0xFFFF0000u);
    x[6] = __uint_as_float(u.w << 16); x[7] = __uint_as_float(u.w & 0xFFFF0000u);
}
__device__ __forceinline__ uint4 pack(const float (&x)[4])
{
    return make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]),
                      __float_as_uint(x[3]));
}
__device__ __forceinline__ uint4 pack(const float (&x)[8])
{
    uint4 u;
    u.x = (uint32_t)f32_to_bf16(x[0]) | ((uint32_t)f32_to_bf16(x[1]) << 16);
    u.y = (uint32_t)f32_to_bf16(x[2]) | ((uint32_t)f32_to_bf16(x[3]) << 16);
    u.z = (uint32_t)f32_to_bf16(x[4]) | ((uint32_t)f32_to_bf16(x[5]) << 16);
    u.w = (uint32_t)f32_to_bf16(x[6]) | ((uint32_t)f32_to_bf16(x[7]) << 16);
    return u;
}

constexpr int ASM_THREADS = 256;

// The tile of this workgroup: which rows of which segment, from where, to where.
struct Tile {
    int64_t k_off, v_ahead;  // elements: first K row of the tile; the V row is v_ahead further on
    int n_tok, dst_row, pos, req, layer, head;
};

__device__ __forceinline__ Tile fetch_tile(const AsmArgs &a, int d)
{
    const int b = (int)blockIdx.x;
    AsmSeg g;
    if (a.segs) {
        g = a.segs[a.tile_seg[b]];  // (wave-uniform)
    } else if (a.seg_tiles > 0) {
        g = a.inline_seg[b / a.seg_tiles];  // packets of one length: no search
    } else {
        int j = 0;
        while (j + 1 < a.n_segs && a.inline_seg[j + 1].tile0 <= b) ++j;
        g = a.inline_seg[j];
    }
    Tile t;
    const int tok0 = (b - g.tile0) * a.tile_rows;
    t.n_tok = g.n_rows - tok0 < a.tile_rows ? g.n_rows - tok0 : a.tile_rows;
    t.dst_row = g.dst_row + tok0;
    t.pos = g.pos;
    t.req = g.req;
    const int lh = (int)blockIdx.y;
    const bool own_layer = g.stride < 0;  // compressed packet: the blob is laid out layer by layer
    const int stride = own_layer ? -g.stride : g.stride;
    t.v_ahead = (int64_t)(own_layer ? 1 : a.n_layers_total) * a.n_kv * stride * d;
    if (a.layered) {
        t.layer = g.layer;
        t.head = lh;
        t.k_off = g.src_base + ((int64_t)t.head * stride + tok0) * d;
    } else {
        t.layer = a.layer_begin + lh / a.n_kv;
        t.head = lh % a.n_kv;
        t.k_off = g.src_base + (((int64_t)t.layer * a.n_kv + t.head) * stride + tok0) * d;
    }
    return t;
}

// Vector path: D (head_dim) is a compile-time power of two with D/2 a multiple of the
// 16-byte vector width, so a thread's column chunk is the same in every pass.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <bool NT> __device__ __forceinline__ uint4 ld16(const void *p)
{
    if (NT) {
        u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
        return make_uint4(v.x, v.y, v.z, v.w);
    }
    return *(const uint4 *)p;
}
template <bool NT> __device__ __forceinline__ void st16(void *p, const uint4 &u)
{
    if (NT) {
        u32x4 v = {u.x, u.y, u.z, u.w};
        __builtin_nontemporal_store(v, (u32x4 *)p);
    } else {
        *(uint4 *)p = u;
    }
}

template <typename T, int D, int ROWS, bool NT>
__global__ __launch_bounds__(ASM_THREADS) void assemble_vec_kernel(AsmArgs a)
{
    constexpr int N = Vec16<T>::N;
    constexpr int HALF = D / 2;
    constexpr int CPR = HALF / N;                  // K: (lo, hi) chunk pairs per row
    constexpr int KROWS = ASM_THREADS / CPR;       // rows per pass
    constexpr int KPASS = (ROWS + KROWS - 1) / KROWS;
    constexpr int VCPR = D / N;                    // V: chunks per row
    constexpr int VROWS = ASM_THREADS / VCPR;
    constexpr int VPASS = (ROWS + VROWS - 1) / VROWS;
    static_assert(CPR >= 1 && ASM_THREADS % CPR == 0 && KPASS >= 1 && VPASS >= 1, "shape");

    const Tile tile = fetch_tile(a, D);
    const int tid = threadIdx.x;
    const int layer = tile.layer, head = tile.head;
    const T *ksrc = (const T *)a.arena + tile.k_off;
    const T *vsrc = ksrc + tile.v_ahead;
    T *kdst = (T *)a.cache.k;
    T *vdst = (T *)a.cache.v;

    // With split_kv a workgroup moves either the K rows or the V rows of its tile: one
    // contiguous source run and one destination run per workgroup (measured on plain copies:
    // 16 KB from one region per workgroup 6.1 TB/s, 8 KB from each of two regions 5.8).
    const bool do_k = !a.split_kv || blockIdx.z == 0, do_v = !a.split_kv || blockIdx.z == 1;

    // issue every load of the tile first
    const int kc = tid % CPR, kr0 = tid / CPR;
    uint4 klo[KPASS], khi[KPASS];
#pragma unroll
    for (int p = 0; p < KPASS; ++p) {
        int r = kr0 + p * KROWS;
        if (do_k && r < tile.n_tok) {
            klo[p] = ld16<NT>(ksrc + (int64_t)r * D + kc * N);
            khi[p] = ld16<NT>(ksrc + (int64_t)r * D + HALF + kc * N);
        }
    }
    const int vc = tid % VCPR, vr0 = tid / VCPR;
    uint4 vv[VPASS];
#pragma unroll
    for (int p = 0; p < VPASS; ++p) {
        int r = vr0 + p * VROWS;
        if (do_v && r < tile.n_tok) vv[p] = ld16<NT>(vsrc + (int64_t)r * D + vc * N);
    }
    float c[N], s[N];
    if (do_k) {
        const float2 *cs = a.cs + (int64_t)tile.pos * HALF + kc * N;
#pragma unroll
        for (int i = 0; i < N; ++i) { float2 t = cs[i]; c[i] = t.x; s[i] = t.y; }
    }

#pragma unroll
    for (int p = 0; p < VPASS; ++p) {
        int r = vr0 + p * VROWS;
        if (do_v && r < tile.n_tok) {
            int64_t o = cache_row_off(a.cache, tile.req, layer, head, tile.dst_row + r, a.n_kv, D);
            st16<NT>(vdst + o + vc * N, vv[p]);
        }
    }
#pragma unroll
    for (int p = 0; p < KPASS; ++p) {
        int r = kr0 + p * KROWS;
        if (do_k && r < tile.n_tok) {
            float x[N], y[N], lo[N], hi[N];
            unpack(klo[p], x);
            unpack(khi[p], y);
#pragma unroll
            for (int i = 0; i < N; ++i) {
                float xc = x[i] * c[i], ys = y[i] * s[i];
                float yc = y[i] * c[i], xs = x[i] * s[i];
                lo[i] = xc - ys;
                hi[i] = yc + xs;
            }
            int64_t o = cache_row_off(a.cache, tile.req, layer, head, tile.dst_row + r, a.n_kv, D);
            st16<NT>(kdst + o + kc * N, pack(lo));
            st16<NT>(kdst + o + HALF + kc * N, pack(hi));
        }
    }
}

// Scalar path for any even head_dim.
template <typename T>
__global__ __launch_bounds__(ASM_THREADS) void assemble_scalar_kernel(AsmArgs a)
{
    const int d = a.d, half = d / 2;
    const Tile tile = fetch_tile(a, d);
    const int layer = tile.layer, head = tile.head;
    const T *ksrc = (const T *)a.arena + tile.k_off;
    const T *vsrc = ksrc + tile.v_ahead;
    T *kdst = (T *)a.cache.k;
    T *vdst = (T *)a.cache.v;
    const float2 *cs = a.cs + (int64_t)tile.pos * half;
    for (int idx = threadIdx.x; idx < tile.n_tok * half; idx += ASM_THREADS) {
        int r = idx / half, i = idx % half;
        float x = ld_elem(ksrc + (int64_t)r * d + i), y = ld_elem(ksrc + (int64_t)r * d + half + i);
        float2 t = cs[i];
        float xc = x * t.x, ys = y * t.y, yc = y * t.x, xs = x * t.y;
        int64_t o = cache_row_off(a.cache, tile.req, layer, head, tile.dst_row + r, a.n_kv, d);
        st_elem(kdst + o + i, xc - ys);
        st_elem(kdst + o + half + i, yc + xs);
        vdst[o + i] = vsrc[(int64_t)r * d + i];
        vdst[o + half + i] = vsrc[(int64_t)r * d + half + i];
    }
}

template <typename T, int D> static void launch_vec(const AsmArgs &a, dim3 grid, hipStream_t st, bool nt)
{
    dim3 block(ASM_THREADS);
#define KVP_ASM_CASE(R)                                                                                   \
    if (nt) hipLaunchKernelGGL((assemble_vec_kernel<T, D, R, true>), grid, block, 0, st, a);              \
    else hipLaunchKernelGGL((assemble_vec_kernel<T, D, R, false>), grid, block, 0, st, a)
    if (a.tile_rows == 16) { KVP_ASM_CASE(16); }
    else if (a.tile_rows == 32) { KVP_ASM_CASE(32); }
    else { KVP_ASM_CASE(64); }
#undef KVP_ASM_CASE
}

int launch_assemble(int dtype, const AsmArgs &a, int n_layers_launch, void *stream)
{
    if (a.n_tiles == 0 || n_layers_launch == 0) return 0;
    if (a.tile_rows != 16 && a.tile_rows != 32 && a.tile_rows != 64) return (int)hipErrorInvalidValue;
    const bool vec = a.d == 64 || a.d == 128 || a.d == 256;
    if (a.split_kv && !vec) return (int)hipErrorInvalidValue;  // (the scalar kernel moves both)
    dim3 grid((unsigned)a.n_tiles, (unsigned)(n_layers_launch * a.n_kv), a.split_kv ? 2u : 1u);
    dim3 block(ASM_THREADS);
    hipStream_t st = (hipStream_t)stream;
    const bool nt = a.nontemporal != 0;
    if (dtype == 1) {
        if (a.d == 128) launch_vec<bf16_t, 128>(a, grid, st, nt);
        else if (a.d == 64) launch_vec<bf16_t, 64>(a, grid, st, nt);
        else if (a.d == 256) launch_vec<bf16_t, 256>(a, grid, st, nt);
        else hipLaunchKernelGGL((assemble_scalar_kernel<bf16_t>), grid, block, 0, st, a);
    } else {
        if (a.d == 128) launch_vec<float, 128>(a, grid, st, nt);
        else if (a.d == 64) launch_vec<float, 64>(a, grid, st, nt);
        else if (a.d == 256) launch_vec<float, 256>(a, grid, st, nt);
        else hipLaunchKernelGGL((assemble_scalar_kernel<float>), grid, block, 0, st, a);
    }
    return (int)hipGetLastError();
}

// A call's plan goes from its pinned host buffer to its device twin through this kernel
// (the device reads host memory directly): next to the launches that follow it on the stream
// it costs a few microseconds, where a copy-engine transfer and its hand-over to the compute
// queue cost some twenty.
__global__ __launch_bounds__(256) void plan_upload_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int n16)
{
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i < n16) dst[i] = src[i];
}

int launch_plan_upload(const void *host, void *dev, uint64_t bytes, void *stream)
{
    const uint64_t n16 = (bytes + 15) / 16;  // plan buffers are sized in multiples of 4 KB
    if (n16 == 0) return 0;
    if (n16 > 0x7fffffffull || (((uintptr_t)host | (uintptr_t)dev) & 15)) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(plan_upload_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)host, (uint4 *)dev, (int)n16);
    return (int)hipGetLastError();
}

}  // namespace kvp
