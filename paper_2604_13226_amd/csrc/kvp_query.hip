// kvp_query.hip -- K2: query-side RoPE + append; generic (any dtype, any head_dim)
// split-KV attention; K4: split-KV combine.  (Sec. 4.2.1 step 4; Fig. 2(d).)
#include "kvp_device.h"

namespace kvp {

// ---------------------------------------------------------------------------------
// K2.  One thread per (query row, head, pair i): rotates Q and K_new from position 0 to
// ctx_len + t, writes the rotated Q to the workspace (store dtype), the rotated K_new and
// the raw V_new to cache rows ctx_len + t.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void append_kernel(AppendArgs a)
{
#pragma clang fp contract(off)
    const int half = a.d / 2;
    const int heads = a.n_q_heads + a.n_kv;
    const int64_t total = (int64_t)a.tot_q * heads * half;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        int i = (int)(idx % half);
        int64_t rh = idx / half;
        int hh = (int)(rh % heads);
        int row = (int)(rh / heads);
        int req = a.row_req[row];
        ReqMeta m = a.reqs[req];
        const int row_in_req = row - m.q_off;
        int pos = m.pos0 + row_in_req;            // the token's position
        const int cache_row = m.ctx_len + row_in_req;  // the cache row its K / V go to
        float c = 1.f, s = 0.f;
        if (!a.prerotated) {
            float2 t = a.cs[(int64_t)pos * half + i];
            c = t.x;
            s = t.y;
        }
        if (hh < a.n_q_heads) {
            int64_t o = ((int64_t)row * a.n_q_heads + hh) * a.d;
            const T *src = (const T *)a.q + o;
            T *dst = (T *)a.q_rot + o;
            float x = ld_elem(src + i), y = ld_elem(src + half + i);
            float xc = x * c, ys = y * s, yc = y * c, xs = x * s;
            st_elem(dst + i, (xc - ys) * a.q_scale);
            st_elem(dst + half + i, (yc + xs) * a.q_scale);
        } else {
            int h = hh - a.n_q_heads;
            int64_t o = ((int64_t)row * a.n_kv + h) * a.d;
            const T *ks = (const T *)a.k_new + o;
            const T *vs = (const T *)a.v_new + o;
            int64_t co = cache_row_off(a.cache, req, a.layer, h, cache_row, a.n_kv, a.d);
            T *kd = (T *)a.cache.k + co;
            T *vd = (T *)a.cache.v + co;
            float x = ld_elem(ks + i), y = ld_elem(ks + half + i);
            float xc = x * c, ys = y * s, yc = y * c, xs = x * s;
            st_elem(kd + i, xc - ys);
            st_elem(kd + half + i, yc + xs);
            vd[i] = vs[i];
            vd[half + i] = vs[half + i];
        }
    }
}

int launch_append(int dtype, const AppendArgs &a, void *stream)
{
    if (a.tot_q == 0) return 0;
    int64_t total = (int64_t)a.tot_q * (a.n_q_heads + a.n_kv) * (a.d / 2);
    unsigned blocks = (unsigned)((total + 255) / 256);
    if (blocks > 65536u) blocks = 65536u;
    if (dtype == 1) hipLaunchKernelGGL((append_kernel<bf16_t>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL((append_kernel<float>), dim3(blocks), dim3(256), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Generic attention: one wavefront per packed row, lanes own head_dim/64 columns
// (head_dim <= 256), online softmax over the item's kv range in fp32.  Slow but
// shape-agnostic: the fp32 path and any shape the MFMA kernel does not take.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <typename T>
__global__ __launch_bounds__(256) void attention_generic_kernel(AttnArgs a)
{
    const AttnItem it = a.items[blockIdx.x];
    if (it.n_rows <= 0) return;  // padding item of the launch order
    const AttnGroup gp = a.groups[it.group];
    const ReqMeta rq = a.reqs[gp.req];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d = a.d;
    const T *kc = (const T *)a.cache.k;
    const T *vc = (const T *)a.cache.v;

    for (int rr = wave; rr < gp.n_rows; rr += 4) {
        const int m = gp.m0 + rr;
        const int t = m / a.g, hq = gp.kv_head * a.g + m % a.g;
        const T *qp = (const T *)a.q_rot + ((int64_t)(rq.q_off + t) * a.n_q_heads + hq) * d;
        float q[4], o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int e = lane + 64 * j;
            q[j] = e < d ? ld_elem(qp + e) : 0.f;
            o[j] = 0.f;
        }
        float mx = -INFINITY, l = 0.f;
        int vis_end = rq.ctx_len + t + 1;  // causal among the query rows, full over the prefix
        int end = it.kv_end < vis_end ? it.kv_end : vis_end;
        // UB rows per trip: all their K and V loads are issued before the first is used, so a
        // trip costs one memory round trip instead of UB
        constexpr int UB = 8;
        for (int u0 = it.kv_begin; u0 < end; u0 += UB) {
            float kk[UB][4], v[UB][4];
#pragma unroll
            for (int i = 0; i < UB; ++i) {
                const int u = u0 + i < end ? u0 + i : end - 1;  // rows past the range repeat the last one (unused)
                const int64_t off = cache_row_off(a.cache, gp.req, a.layer, gp.kv_head, u, a.n_kv, d);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = lane + 64 * j;
                    kk[i][j] = e < d ? ld_elem(kc + off + e) : 0.f;
                    v[i][j] = e < d ? ld_elem(vc + off + e) : 0.f;
                }
            }
#pragma unroll
            for (int i = 0; i < UB; ++i) {
                if (u0 + i >= end) break;  // wave-uniform
                float part = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) part += q[j] * kk[i][j];
                float sc = wave_sum(part) * a.scale_log2e;
                float mn = fmaxf(mx, sc);
                float alpha = exp2f(mx - mn);  // exp2f(-inf) = 0 on the first row
                float p = exp2f(sc - mn);
                l = l * alpha + p;
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = o[j] * alpha + p * v[i][j];
                mx = mn;
            }
        }
        if (gp.n_splits == 1) {
            T *op = (T *)a.out + ((int64_t)(rq.q_off + t) * a.n_q_heads + hq) * d;
            float inv = 1.f / l;  // the row always sees itself, so l > 0
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int e = lane + 64 * j;
                if (e < d) st_elem(op + e, o[j] * inv);
            }
        } else {
            float *pp = (float *)((char *)a.partials + (int64_t)(gp.part0 + it.split) * part_slot_bytes(a.bm, d, 0));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int e = lane + 64 * j;
                if (e < d) pp[(int64_t)rr * d + e] = o[j];
            }
            if (lane == 0) {
                pp[(int64_t)a.bm * d + rr] = mx;
                pp[(int64_t)a.bm * d + a.bm + rr] = l;
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// K4.  Merge the splits of one group by log-sum-exp:
//   m = max m_i;  l = sum l_i 2^(m_i - m);  O = sum O~_i 2^(m_i - m) / l.
// A split that saw no visible row has m_i = -inf, l_i = 0 and contributes nothing.
// ---------------------------------------------------------------------------------
// Two shapes.  Many splits per group (the latency-bound single-request calls):
// One wavefront per packed row.  Lane i first holds the log-sum-exp weight of split i (at
// most 64 splits); then lane half hf = i / 32 sweeps the splits of its parity, columns
// 4 (i % 32) .. +3 (+128 j) with 16-byte loads, several splits in flight at once, and the
// two halves are added with one exchange.
constexpr int COMBINE_ROWS = 4;  // rows per 256-thread workgroup

// Four neighbouring columns of a partial row: fp32 as they are, or fp16 (the MFMA kernel's rows,
// scaled per row by a power of two that their m and l carry along) widened.
// A piece stays as loaded (raw) until it is used: widening it right behind its load would put a
// wait behind every load and serialise the memory round trips.
typedef _Float16 halfx4_t __attribute__((ext_vector_type(4)));
template <typename P> struct Part4;
template <> struct Part4<float> { typedef float4 raw; };
template <> struct Part4<_Float16> { typedef uint2 raw; };
__device__ __forceinline__ float4 ld_raw4(const float *p) { return *(const float4 *)p; }
__device__ __forceinline__ uint2 ld_raw4(const _Float16 *p) { return *(const uint2 *)p; }
__device__ __forceinline__ float4 widen4(const float4 &v) { return v; }
__device__ __forceinline__ float4 widen4(const uint2 &u)
{
    const halfx4_t v = __builtin_bit_cast(halfx4_t, u);
    return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}
__device__ __forceinline__ void zero_raw(float4 &v) { v = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void zero_raw(uint2 &v) { v = make_uint2(0u, 0u); }
__device__ __forceinline__ float ld_part1(const float *p) { return *p; }
__device__ __forceinline__ float ld_part1(const _Float16 *p) { return (float)*p; }

template <typename T, typename P, int EARLY>  // EARLY: 4-column loads per lane issued up front (2 EARLY splits of 128 columns)
__global__ __launch_bounds__(256) void combine_wave_kernel(AttnArgs a)
{
    const int lane = threadIdx.x & 63, li = lane & 31, hf = lane >> 5;
    const int rr = (int)blockIdx.y * COMBINE_ROWS + (threadIdx.x >> 6);
    const int d = a.d, stride = a.part_stride;
    const int64_t slot_b = part_slot_bytes(a.bm, d, sizeof(P) == 2);
    const int64_t slot = slot_b / (int64_t)sizeof(P), slot_f = slot_b / 4;  // in row elements / in floats
    // Group gi's partial slots start at gi * stride, so the first loads below do not wait for
    // the group's record; slots and rows the group does not use hold stale bytes of the
    // workspace (in bounds) and are masked once the record has arrived.
    const char *base = (const char *)a.partials + (int64_t)blockIdx.x * stride * slot_b;
    const float *ml = (const float *)(base + part_rows_bytes(a.bm, d, sizeof(P) == 2)) + rr;
    // (loads are unconditional, from addresses clamped into the group's slots: a piece that is not
    // needed is dropped by its weight, and no load waits for a branch to rejoin)
    const P *row = (const P *)base + (int64_t)(rr < a.bm ? rr : a.bm - 1) * d;
    constexpr int BATCH = 8;   // later loads go out BATCH per lane at a time, all before the first is used
    const int col0 = (d & 3) == 0 ? (4 * li < d ? 4 * li : d - 4) : 0;
    typename Part4<P>::raw v0[EARLY];
    if ((d & 3) == 0) {
#pragma unroll
        for (int i = 0; i < EARLY; ++i) {
            const int sq = 2 * i + hf;
            v0[i] = ld_raw4(row + (sq < stride ? sq : stride - 1) * slot + col0);
        }
    } else {
#pragma unroll
        for (int i = 0; i < EARLY; ++i) zero_raw(v0[i]);
    }
    float mi = -INFINITY, lv = 0.f;
    if (lane < stride && rr < a.bm) { mi = ml[lane * slot_f]; lv = ml[lane * slot_f + a.bm]; }
    const AttnGroup gp = a.groups[blockIdx.x];
    const int ns = gp.n_splits;
    if (ns <= 1 || rr >= gp.n_rows) return;
    if (lane >= ns) { mi = -INFINITY; lv = 0.f; }
    float mx = mi;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    const float w = (mi == -INFINITY) ? 0.f : exp2f(mi - mx);
    const float inv = 1.f / wave_sum(lv * w);
    const int m = gp.m0 + rr;
    const int t = m / a.g, hq = gp.kv_head * a.g + m % a.g;
    T *op = (T *)a.out + ((int64_t)(gp.q_off + t) * a.n_q_heads + hq) * d;
    // Every lane runs every trip of the loops below (the weights travel by lane shuffles, which
    // need their source lanes active); `on` guards the loads and stores of lanes past the row.
    if ((d & 3) == 0) {
        for (int e0 = 0; e0 < d; e0 += 128) {
            const int e = e0 + 4 * li;
            const bool on = e < d;
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            int s_from = 0;
            if (e0 == 0) {  // the pieces already on their way
#pragma unroll
                for (int i = 0; i < EARLY; ++i) {
                    const int sq = 2 * i + hf, sp = sq < ns ? sq : ns - 1;
                    const float ws = __shfl(w, sp, 64);
                    // (a split without visible rows has weight 0 and may hold anything)
                    const float4 v = widen4(v0[i]);
                    if (sq < ns && ws != 0.f) { acc.x += v.x * ws; acc.y += v.y * ws; acc.z += v.z * ws; acc.w += v.w * ws; }
                }
                s_from = 2 * EARLY;
            }
            // (a loop that loads one piece per trip waits a memory round trip per trip: with 22
            // splits its three last trips cost 2 us)
            for (int s2 = s_from; s2 < ns; s2 += 2 * BATCH) {  // same trip count in both halves
                typename Part4<P>::raw vr[BATCH];
#pragma unroll
                for (int i = 0; i < BATCH; ++i) {
                    const int sq = s2 + 2 * i + hf;
                    vr[i] = ld_raw4(row + (sq < ns ? sq : ns - 1) * slot + (on ? e : d - 4));
                }
#pragma unroll
                for (int i = 0; i < BATCH; ++i) {
                    const int sq = s2 + 2 * i + hf, sp = sq < ns ? sq : ns - 1;
                    float ws = __shfl(w, sp, 64);
                    if (sq >= ns) ws = 0.f;
                    const float4 v = widen4(vr[i]);
                    if (ws != 0.f) { acc.x += v.x * ws; acc.y += v.y * ws; acc.z += v.z * ws; acc.w += v.w * ws; }
                }
            }
            acc.x += __shfl_xor(acc.x, 32, 64);
            acc.y += __shfl_xor(acc.y, 32, 64);
            acc.z += __shfl_xor(acc.z, 32, 64);
            acc.w += __shfl_xor(acc.w, 32, 64);
            if (hf == 0 && on) {
                st_elem(op + e, acc.x * inv);
                st_elem(op + e + 1, acc.y * inv);
                st_elem(op + e + 2, acc.z * inv);
                st_elem(op + e + 3, acc.w * inv);
            }
        }
    } else {
        for (int e0 = 0; e0 < d; e0 += 64) {
            const int e = e0 + lane;
            const bool on = e < d;
            float acc = 0.f;
            for (int sp = 0; sp < ns; ++sp) {
                const float ws = __shfl(w, sp, 64);
                if (on && ws != 0.f) acc += ld_part1(row + sp * slot + e) * ws;
            }
            if (on) st_elem(op + e, acc * inv);
        }
    }
}

// Few splits per group (at most COMBINE_EARLY: the batched calls, where rows are many):
// One thread per (row, column chunk): VW columns of one packed row, so a 256-thread workgroup
// covers 256 VW / d rows.  The threads of a row first put the (m, l) of its splits into LDS
// (one load each) while every thread already has the O pieces of the first EARLY splits on
// their way -- group gi's partial slots start at gi * part_stride, so none of these loads waits
// for the group's record; slots and rows the group does not use hold stale bytes of the
// workspace (in bounds) and are masked once the record is there.  Then each thread merges its
// own columns: no exchange between lanes.
constexpr int COMBINE_EARLY = 8;
constexpr int COMBINE_MAX_SPLITS = 64;  // the planner's bound on splits per group
__host__ __device__ inline int combine_rows_per_block(int cpr) { int r = 256 / cpr; return r > 32 ? 32 : r; }

template <int VW> struct CombineVec;
template <> struct CombineVec<4> { typedef float4 type; };
template <> struct CombineVec<1> { typedef float type; };

__device__ __forceinline__ void cv_fma(float4 &acc, const float4 &v, float w) { acc.x += v.x * w; acc.y += v.y * w; acc.z += v.z * w; acc.w += v.w * w; }
__device__ __forceinline__ void cv_fma(float &acc, const float &v, float w) { acc += v * w; }
__device__ __forceinline__ void cv_zero(float4 &v) { v = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void cv_zero(float &v) { v = 0.f; }
// raw piece types of the thread kernel: VW = 4 as above, VW = 1 a single fp32 / fp16 value
template <typename P, int VW> struct RawVec { typedef typename Part4<P>::raw type; };
template <> struct RawVec<float, 1> { typedef float type; };
template <> struct RawVec<_Float16, 1> { typedef _Float16 type; };
__device__ __forceinline__ void cv_load_raw(float4 &v, const float *p) { v = ld_raw4(p); }
__device__ __forceinline__ void cv_load_raw(uint2 &v, const _Float16 *p) { v = ld_raw4(p); }
__device__ __forceinline__ void cv_load_raw(float &v, const float *p) { v = *p; }
__device__ __forceinline__ void cv_load_raw(_Float16 &v, const _Float16 *p) { v = *p; }
__device__ __forceinline__ void zero_raw(float &v) { v = 0.f; }
__device__ __forceinline__ void zero_raw(_Float16 &v) { v = (_Float16)0.f; }
__device__ __forceinline__ float widen(const float &v) { return v; }
__device__ __forceinline__ float widen(const _Float16 &v) { return (float)v; }
__device__ __forceinline__ float4 widen(const float4 &v) { return v; }
__device__ __forceinline__ float4 widen(const uint2 &v) { return widen4(v); }
template <typename T> __device__ __forceinline__ void cv_store(T *p, const float4 &v, float s)
{
    st_elem(p, v.x * s); st_elem(p + 1, v.y * s); st_elem(p + 2, v.z * s); st_elem(p + 3, v.w * s);
}
template <typename T> __device__ __forceinline__ void cv_store(T *p, const float &v, float s) { st_elem(p, v * s); }

template <typename T, typename P, int VW>
__global__ __launch_bounds__(256) void combine_thread_kernel(AttnArgs a)
{
    typedef typename CombineVec<VW>::type vec_t;
    extern __shared__ float ml_lds[];  // [rows per block][2][stride]
    const int d = a.d, cpr = d / VW;   // chunks (threads) per row
    const int rpb = combine_rows_per_block(cpr);
    const int rb = (int)threadIdx.x / cpr, c = (int)threadIdx.x % cpr;
    const bool active = rb < rpb;      // threads beyond the block's last whole row only keep the barrier company
    const int rr = active ? (int)blockIdx.y * rpb + rb : a.bm;
    const int stride = a.part_stride;
    const int64_t slot_b = part_slot_bytes(a.bm, d, sizeof(P) == 2);
    const int64_t slot = slot_b / (int64_t)sizeof(P), slot_f = slot_b / 4;  // in row elements / in floats
    const char *base = (const char *)a.partials + (int64_t)blockIdx.x * stride * slot_b;
    const bool in_slot = rr < a.bm;
    const float *ml = (const float *)(base + part_rows_bytes(a.bm, d, sizeof(P) == 2)) + rr;
    const P *row = (const P *)base + (int64_t)rr * d + c * VW;

    typedef typename RawVec<P, VW>::type raw_t;
    raw_t v0[COMBINE_EARLY];
#pragma unroll
    for (int i = 0; i < COMBINE_EARLY; ++i) {
        zero_raw(v0[i]);
        if (in_slot && i < stride) cv_load_raw(v0[i], row + i * slot);
    }
    float *my_m = ml_lds + ((active ? rb : 0) * 2) * stride, *my_l = my_m + stride;
    for (int sp = c; active && sp < stride; sp += cpr) {
        my_m[sp] = in_slot ? ml[sp * slot_f] : -INFINITY;
        my_l[sp] = in_slot ? ml[sp * slot_f + a.bm] : 0.f;
    }
    const AttnGroup gp = a.groups[blockIdx.x];
    __syncthreads();
    const int ns = gp.n_splits;
    if (ns <= 1 || rr >= gp.n_rows) return;
    float mx = -INFINITY;
    for (int sp = 0; sp < ns; ++sp) mx = fmaxf(mx, my_m[sp]);
    vec_t acc;
    cv_zero(acc);
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < COMBINE_EARLY; ++i)
        if (i < ns) {
            const float mi = my_m[i];
            const float w = mi == -INFINITY ? 0.f : exp2f(mi - mx);
            lsum += my_l[i] * w;
            if (w != 0.f) cv_fma(acc, widen(v0[i]), w);  // a split without visible rows may hold anything
        }
#pragma unroll 4
    for (int sp = COMBINE_EARLY; sp < ns; ++sp) {
        const float mi = my_m[sp];
        const float w = mi == -INFINITY ? 0.f : exp2f(mi - mx);
        lsum += my_l[sp] * w;
        raw_t v;
        cv_load_raw(v, row + sp * slot);
        if (w != 0.f) cv_fma(acc, widen(v), w);
    }
    const int m = gp.m0 + rr;
    const int t = m / a.g, hq = gp.kv_head * a.g + m % a.g;
    T *op = (T *)a.out + ((int64_t)(gp.q_off + t) * a.n_q_heads + hq) * d + c * VW;
    cv_store(op, acc, 1.f / lsum);
}

template <typename T, typename P> static void launch_combine_typed(const AttnArgs &a, int rows, hipStream_t st)
{
    if (a.part_stride > COMBINE_EARLY) {  // many splits: a wavefront per row, its lanes over the splits
        dim3 grid((unsigned)a.n_groups, (unsigned)((rows + COMBINE_ROWS - 1) / COMBINE_ROWS));
        // up to 16 splits: 8 early loads per lane cover them; more: 12, so that the 19-24 splits of
        // a single 8K request still take one memory round trip (measured per layer: 8K 22.5 -> 22.0 us,
        // one decode step over it 17.5 -> 16.9; with 12 splits the larger kernel is 0.2 us slower)
        // (... and 16 / 20 for up to 32 / 40 splits: a second round trip costs 2 us)
        if (a.part_stride <= 16) hipLaunchKernelGGL((combine_wave_kernel<T, P, 8>), grid, dim3(256), 0, st, a);
        else if (a.part_stride <= 24) hipLaunchKernelGGL((combine_wave_kernel<T, P, 12>), grid, dim3(256), 0, st, a);
        else if (a.part_stride <= 32) hipLaunchKernelGGL((combine_wave_kernel<T, P, 16>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((combine_wave_kernel<T, P, 20>), grid, dim3(256), 0, st, a);
        return;
    }
    const int vw = a.d % 4 == 0 ? 4 : 1;
    const int cpr = a.d / vw;
    const int rpb = combine_rows_per_block(cpr);
    dim3 grid((unsigned)a.n_groups, (unsigned)((rows + rpb - 1) / rpb));
    const size_t lds = (size_t)rpb * 2 * a.part_stride * sizeof(float);
    if (vw == 4) hipLaunchKernelGGL((combine_thread_kernel<T, P, 4>), grid, dim3(256), lds, st, a);
    else hipLaunchKernelGGL((combine_thread_kernel<T, P, 1>), grid, dim3(256), lds, st, a);
}

int launch_combine(int dtype, const AttnArgs &a, void *stream)
{
    if (a.n_groups == 0) return 0;
    const int rows = a.max_group_rows > 0 && a.max_group_rows < a.bm ? a.max_group_rows : a.bm;
    hipStream_t st = (hipStream_t)stream;
    if (a.part_stride > COMBINE_MAX_SPLITS) return (int)hipErrorInvalidValue;
    const int cpr = a.d / (a.d % 4 == 0 ? 4 : 1);
    if (cpr < 1 || cpr > 256) return (int)hipErrorInvalidValue;
    if (a.part_f16) {  // the MFMA kernel's partial rows (bf16 stores only)
        if (dtype != 1 || (a.d & 3)) return (int)hipErrorInvalidValue;
        launch_combine_typed<bf16_t, _Float16>(a, rows, st);
    } else if (dtype == 1) {
        launch_combine_typed<bf16_t, float>(a, rows, st);
    } else {
        launch_combine_typed<float, float>(a, rows, st);
    }
    return (int)hipGetLastError();
}

int launch_attention_mfma(const AttnArgs &a, void *stream);  // kvp_attention_mfma.hip

int launch_attention(int dtype, const AttnArgs &a, int kernel_kind, void *stream)
{
    if (a.n_items == 0) return 0;
    if (kernel_kind == ATTN_MFMA) return launch_attention_mfma(a, stream);
    if (dtype == 1) hipLaunchKernelGGL((attention_generic_kernel<bf16_t>), dim3(a.n_items), dim3(256), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL((attention_generic_kernel<float>), dim3(a.n_items), dim3(256), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

}  // namespace kvp
