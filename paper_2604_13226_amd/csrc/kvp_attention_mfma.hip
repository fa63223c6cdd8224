// kvp_attention_mfma.hip -- K3: query-prefill attention on the bf16 matrix cores
// (Sec. 4.2.1 step 4; Fig. 2(d): full over the packet prefix, causal among the query rows).
//
// One workgroup = 4 wavefronts = one work item: rows [m0, m0+128) of the packed
// (query token, query head) rows that share one KV head, over one kv range (split-KV).
// Wave w owns 32 rows.  Per 64-row K/V tile, staged once through LDS for all 128 rows:
//
//   S^T = K Q^T      v_mfma_f32_32x32x16_bf16, A = K tile rows from LDS (16-byte reads),
//                    B = Q^T held in registers for the whole item
//   online softmax   a lane owns one query row (column of S^T): row max / row sum are
//                    in-lane reductions plus one exchange with lane ^ 32
//   O^T += V^T P^T   A = V^T read straight out of the row-major V tile with the
//                    transposing LDS read (ds_read_b64_tr_b16), B = P^T taken from the
//                    S^T accumulators in place: the kv order inside each 16-row k-step is
//                    whatever the accumulator layout gives, applied to both operands.
//
// HBM traffic: every K/V row of the range is read once per group of 128 packed rows.
#include "kvp_device.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;          // packed rows per workgroup
constexpr int BN = 64;           // kv rows per tile
constexpr int D = 128;           // head_dim
constexpr int K_STRIDE = D + 8;  // LDS row strides (elements): 272 B and 320 B keep the
constexpr int V_STRIDE = D + 32; // 16-byte K reads and the transposing V reads conflict-free
constexpr int K_TILE = BN * K_STRIDE;
constexpr int V_TILE = BN * V_STRIDE;
constexpr int LDS_BYTES = 2 * (K_TILE + V_TILE) * 2;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

__global__ __launch_bounds__(256, 2) void attention_mfma_kernel(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    const AttnItem it = a.items[blockIdx.x];
    const AttnGroup gp = a.groups[it.group];
    const ReqMeta rq = a.reqs[gp.req];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int g = a.g;

    // this lane's query row
    const int rr = 32 * wave + n;
    const bool row_ok = rr < gp.n_rows;
    const int m = gp.m0 + (row_ok ? rr : 0);
    const int t = m / g, hq = gp.kv_head * g + m % g;
    const int limit = row_ok ? rq.ctx_len + t + 1 : 0;  // kv rows [0, limit) are visible

    // B operand of S^T = K Q^T: lane holds Q[m][16 ks + 8 h .. +7] for ks = 0..7
    bf16x8 qf[8];
    {
        const bf16_t *qp = (const bf16_t *)a.q_rot + ((int64_t)(rq.q_off + t) * a.n_q_heads + hq) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 u = row_ok ? *(const uint4 *)(qp + 16 * ks) : make_uint4(0, 0, 0, 0);
            qf[ks] = __builtin_bit_cast(bf16x8, u);
        }
    }

    floatx16 oacc[4];
#pragma unroll
    for (int eb = 0; eb < 4; ++eb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[eb][r] = 0.f;
    float m_i = -INFINITY, l_i = 0.f;

    const bf16_t *kc = (const bf16_t *)a.cache.k;
    const bf16_t *vc = (const bf16_t *)a.cache.v;
    // staging: thread copies 16-byte chunk (tid % 16) of tile rows tid / 16 + 16 i
    const int ld_row = tid >> 4, ld_chunk = tid & 15;
    uint4 kreg[4], vreg[4];
    auto fetch = [&](int kv0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int kv = kv0 + ld_row + 16 * i;
            if (kv < it.kv_end) {
                int64_t off = cache_row_off(a.cache, gp.req, a.layer, gp.kv_head, kv, a.n_kv, D) + 8 * ld_chunk;
                kreg[i] = *(const uint4 *)(kc + off);
                vreg[i] = *(const uint4 *)(vc + off);
            } else {  // rows past the range: zeros, so masked probabilities meet finite values
                kreg[i] = make_uint4(0, 0, 0, 0);
                vreg[i] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto stage = [&](int buf) {
        bf16_t *kl = lds + buf * (K_TILE + V_TILE);
        bf16_t *vl = kl + K_TILE;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int row = ld_row + 16 * i;
            *(uint4 *)(kl + row * K_STRIDE + 8 * ld_chunk) = kreg[i];
            *(uint4 *)(vl + row * V_STRIDE + 8 * ld_chunk) = vreg[i];
        }
    };

    const int n_tiles = (it.kv_end - it.kv_begin + BN - 1) / BN;
    if (n_tiles > 0) {
        fetch(it.kv_begin);
        stage(0);
    }
    __syncthreads();

    for (int ti = 0; ti < n_tiles; ++ti) {
        const int kv0 = it.kv_begin + ti * BN;
        const int buf = ti & 1;
        if (ti + 1 < n_tiles) fetch(kv0 + BN);
        const bf16_t *kl = lds + buf * (K_TILE + V_TILE);
        const bf16_t *vl = kl + K_TILE;

        // ---- S^T = K Q^T : 2 blocks of 32 kv rows x 32 query rows
        floatx16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
            const bf16_t *kp = kl + (32 * kb + n) * K_STRIDE + 8 * h;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                bf16x8 af = __builtin_bit_cast(bf16x8, *(const uint4 *)(kp + 16 * ks));
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, qf[ks], sacc[kb], 0, 0, 0);
            }
        }

        // ---- online softmax; accumulator r of block kb is kv row kv0 + 32 kb + 8 (r/4) + 4 h + r%4
        const int tile_end = kv0 + BN < it.kv_end ? kv0 + BN : it.kv_end;
        const bool need_mask = tile_end > limit || kv0 + BN > it.kv_end;
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float s = sacc[kb][r] * a.scale_log2e;
                if (need_mask) {
                    int kv = kv0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (kv >= limit || kv >= it.kv_end) s = -INFINITY;
                }
                sacc[kb][r] = s;
                mx = fmaxf(mx, s);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_i, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;  // nothing visible yet: p = 0
        const float alpha = exp2f(m_i - m_use);
        float rs = 0.f;
        uint32_t pk[2][8];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                float p0 = exp2f(sacc[kb][r] - m_use), p1 = exp2f(sacc[kb][r + 1] - m_use);
                rs += p0 + p1;
                pk[kb][r >> 1] = pack_bf16(p0, p1);
            }
        rs += __shfl_xor(rs, 32, 64);
        l_i = l_i * alpha + rs;
        m_i = m_new;
        if (alpha != 1.f) {
#pragma unroll
            for (int eb = 0; eb < 4; ++eb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[eb][r] *= alpha;
        }

        // ---- O^T += V^T P^T.  k-step j of block kb covers kv rows 32 kb + 16 j + [0, 16);
        // P^T slots 0..7 of lane-half h are rows 4h+{0..3} and 8+4h+{0..3} of that step, so
        // the two transposing reads fetch exactly those rows of V for column 32 eb + n.
        const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint4 pu = make_uint4(pk[kb][4 * j], pk[kb][4 * j + 1], pk[kb][4 * j + 2], pk[kb][4 * j + 3]);
                bf16x8 pf = __builtin_bit_cast(bf16x8, pu);
                const bf16_t *vp = vl + (32 * kb + 16 * j + 4 * h + tr_row) * V_STRIDE + tr_col;
#pragma unroll
                for (int eb = 0; eb < 4; ++eb) {
                    typedef __attribute__((address_space(3))) short4v *lds_p;
                    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(vp + 32 * eb));
                    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(vp + 8 * V_STRIDE + 32 * eb));
                    union { short4v s[2]; bf16x8 v; } vf;
                    vf.s[0] = lo;
                    vf.s[1] = hi;
                    oacc[eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf, oacc[eb], 0, 0, 0);
                }
            }

        if (ti + 1 < n_tiles) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds O[m][32 eb + 8 (r/4) + 4 h + r%4]
    if (!row_ok) return;
    if (gp.n_splits == 1) {
        bf16_t *op = (bf16_t *)a.out + ((int64_t)(rq.q_off + t) * a.n_q_heads + hq) * D;
        const float inv = 1.f / l_i;
#pragma unroll
        for (int eb = 0; eb < 4; ++eb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                uint2 u;
                u.x = pack_bf16(oacc[eb][4 * q4] * inv, oacc[eb][4 * q4 + 1] * inv);
                u.y = pack_bf16(oacc[eb][4 * q4 + 2] * inv, oacc[eb][4 * q4 + 3] * inv);
                *(uint2 *)(op + 32 * eb + 8 * q4 + 4 * h) = u;
            }
    } else {
        float *pp = a.partials + (int64_t)(gp.part0 + it.split) * BM * (D + 2);
#pragma unroll
        for (int eb = 0; eb < 4; ++eb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float4 f = make_float4(oacc[eb][4 * q4], oacc[eb][4 * q4 + 1], oacc[eb][4 * q4 + 2], oacc[eb][4 * q4 + 3]);
                *(float4 *)(pp + (int64_t)rr * D + 32 * eb + 8 * q4 + 4 * h) = f;
            }
        if (h == 0) {
            pp[BM * D + rr] = m_i;
            pp[BM * D + BM + rr] = l_i;
        }
    }
}

int launch_attention_mfma(const AttnArgs &a, void *stream)
{
    if (a.d != D || a.bm != BM) return (int)hipErrorInvalidValue;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)attention_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    hipLaunchKernelGGL(attention_mfma_kernel, dim3(a.n_items), dim3(256), LDS_BYTES, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

}  // namespace kvp
