// kvp_attention_mfma.hip -- K3: query-prefill attention on the bf16 matrix cores
// (Sec. 4.2.1 step 4; Fig. 2(d): full over the packet prefix, causal among the query rows).
//
// One workgroup = 4 wavefronts = one work item: rows [m0, m0+128) of the packed
// (query token, query head) rows that share one KV head, over one kv range (split-KV).
// Wave w owns 32 rows.  K/V tiles of 64 rows travel HBM -> LDS directly
// (global_load_lds_dwordx4, no staging registers) through a ring of STAGES tiles, so
// STAGES-1 tiles are in flight while one is being consumed.  Per tile:
//
//   S^T = K Q^T      v_mfma_f32_32x32x16_bf16, A = K rows from LDS (16-byte reads),
//                    B = Q^T held in registers for the whole item
//   online softmax   a lane owns one query row (a column of S^T): row max / row sum are
//                    in-lane reductions plus one exchange with lane ^ 32
//   O^T += V^T P^T   A = V^T read out of the row-major V tile with the transposing LDS
//                    read (ds_read_b64_tr_b16), B = P^T taken from the S^T accumulators in
//                    place: the kv order inside each 16-row k-step is whatever the
//                    accumulator layout gives, applied to both operands.
//
// LDS tiles are unpadded (a direct load writes 64 lanes x 16 B contiguously); bank
// conflicts are avoided by choosing WHICH 16-byte chunk of a row each lane fetches:
// K row r keeps logical chunk c at physical chunk c ^ (r & 15), V row r at c ^ 4 (r & 3).
//
// The kernel also does the query side of the layer (Sec. 4.2.1 step 4): every workgroup
// rotates its own 128 query rows to positions ctx_len + t in registers (the RoPE partner of
// element e is e + 64, which the MFMA operand layout keeps in the same lane), and the
// workgroups whose kv range reaches into the query rows first rotate K_new, write it and
// V_new to the cache rows ctx_len + t, and only then start loading tiles.  Several
// workgroups may write the same rows: they write the same bytes.
//
// HBM traffic: every K/V row of the range is read once per group of 128 packed rows.
#include "kvp_device.h"

namespace kvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void *lds_void_p;
typedef __attribute__((address_space(1))) const void *glb_void_p;

constexpr int BN = 64;   // kv rows per tile
constexpr int D = 128;   // head_dim
constexpr int ROW_BYTES = D * 2;
constexpr int TILE_BYTES = BN * ROW_BYTES;   // 16 KiB for K, same for V
constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // K tile then V tile
constexpr int MAX_BLOCK_IDS = MFMA_MAX_ITEM_BLOCKS;  // paged: block ids of one item kept in LDS

__device__ __forceinline__ uint32_t pack_bf16_hw(float a, float b)
{
    floatx2 f = {a, b};
    bf16x2 v = __builtin_convertvector(f, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, v);
}

// wait until at most n of this wave's vector-memory operations are outstanding
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// x of lane l and of lane l ^ 32, without a trip through the LDS crossbar: the half-swap
// leaves lanes 0..31 of the first result with x[l], of the second with x[l + 32], and the
// upper lanes with the same pair.  The second operand is made opaque to the compiler: given
// the same value twice it was seen to use the first result for both.
__device__ __forceinline__ void xhalf_pair(float x, float &lo, float &hi)
{
    uint32_t u = __builtin_bit_cast(uint32_t, x), w = u;
    asm volatile("" : "+v"(w));
    const auto r = __builtin_amdgcn_permlane32_swap(u, w, false, false);
    uint32_t r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    lo = __builtin_bit_cast(float, r0);
    hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float xhalf_max(float x)
{
    float lo, hi;
    xhalf_pair(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float xhalf_sum(float x)
{
    float lo, hi;
    xhalf_pair(x, lo, hi);
    return lo + hi;
}
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// HBM -> LDS without staging registers: each lane names its own 16 global bytes (a
// wave-uniform base plus a per-lane 32-bit byte offset); the wavefront's 64 x 16 B land
// contiguously at the wave-uniform LDS byte address lds_addr.  Written as inline assembly so
// that the compiler's wait-count insertion does not treat every later LDS read as dependent
// on every outstanding load: the waits are explicit (wait_vmcnt + wg_barrier) in the loop.
// `stream`: the rows will not be read again soon by anyone (no other work item shares them
// through the L2): the load carries the non-temporal hint, which a plain streaming read of HBM
// was measured to reward with 7.0 instead of 6.3 TB/s.
// (A compile-time choice: selected at run time, every load became a branch between two copies of
// the instruction, and the tile loads could no longer be issued between the matrix instructions.)
template <bool STREAM>
__device__ __forceinline__ void load_to_lds_16(const void *sbase, uint32_t voff, uint32_t lds_addr)
{
    if (STREAM)
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
// A 16-byte global load whose wait is ours to place: before the first use of a load it knows,
// the compiler waits for every load issued up to there, the tile loads included (it cannot
// count those), so the query-side loads are made opaque to it as well and waited for by count.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t load16_nowait(const void *p)
{
    u32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
    return v;
}
// a pointer the program knows to be wave-uniform, made so for the compiler too
__device__ __forceinline__ const char *uniform_ptr(const void *p)
{
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
// same with a full per-lane address
__device__ __forceinline__ void load_to_lds_16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}

// If the running reference maximum lags the true row maximum by at most this many
// powers of two, the accumulators are not rescaled (probabilities then reach at most 2^8,
// harmless in fp32 accumulators and scale-free in bf16); the final (m, l, O) stay consistent
// because all three are relative to the same reference.
constexpr float RESCALE_SLACK = 8.f;

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// One 16-byte chunk pair of a head vector rotated by the (cos, sin) pairs in cs4 (Eq. 1):
// element i of the low chunk pairs with element i of the high chunk.
template <bool EXACT>
__device__ __forceinline__ void rotate_chunk_pair(const uint4 &ulo, const uint4 &uhi, const float4 (&cs4)[4], float sign,
                                                  float scale, uint4 &olo, uint4 &ohi)
{
#pragma clang fp contract(off)  // EXACT: separately rounded products and sums, as the gather kernel
    const uint32_t wl[4] = {ulo.x, ulo.y, ulo.z, ulo.w}, wh[4] = {uhi.x, uhi.y, uhi.z, uhi.w};
    uint32_t ol[4], oh[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float lo2[2], hi2[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const float x = __uint_as_float(u ? (wl[j] & 0xFFFF0000u) : (wl[j] << 16));
            const float y = __uint_as_float(u ? (wh[j] & 0xFFFF0000u) : (wh[j] << 16));
            const float c = u ? cs4[j].z : cs4[j].x, sn = (u ? cs4[j].w : cs4[j].y) * sign;
            const float xc = x * c, ys = y * sn, yc = y * c, xs = x * sn;
            lo2[u] = xc - ys;
            hi2[u] = yc + xs;
            if (!EXACT) { lo2[u] *= scale; hi2[u] *= scale; }
        }
        if (EXACT) {
            ol[j] = (uint32_t)f32_to_bf16(lo2[0]) | ((uint32_t)f32_to_bf16(lo2[1]) << 16);
            oh[j] = (uint32_t)f32_to_bf16(hi2[0]) | ((uint32_t)f32_to_bf16(hi2[1]) << 16);
        } else {
            ol[j] = pack_bf16_hw(lo2[0], lo2[1]);
            oh[j] = pack_bf16_hw(hi2[0], hi2[1]);
        }
    }
    olo = make_uint4(ol[0], ol[1], ol[2], ol[3]);
    ohi = make_uint4(oh[0], oh[1], oh[2], oh[3]);
}

enum { SRC_CONTIG = 0, SRC_PAGED = 1, SRC_PACKETS = 2 };

// A tile record of the in-place path, read through the scalar cache: the records are written by
// the host before the launch and never by a kernel, and the index is the same in every lane.  (As
// an ordinary load this was a vector load, and the wait for it -- placed by the compiler, who cannot
// count the tile loads in flight -- drained the whole prefetch ring at every tile.)
__device__ __forceinline__ AttnTile load_tile_record(const AttnTile *tiles, int idx)
{
    typedef const __attribute__((address_space(4))) int32_t *const_i32_p;
    const_i32_p p = (const_i32_p)(uintptr_t)(tiles + __builtin_amdgcn_readfirstlane(idx));
    int32_t w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = p[i];
    AttnTile t;
    __builtin_memcpy(&t, w, sizeof t);
    return t;
}
static_assert(sizeof(AttnTile) == 8 * sizeof(int32_t), "eight words");

// A micro-benchmark that includes this file with -DKVP_TIMING gets per-workgroup time stamps and
// per-wave phase totals through two file-scope pointers it sets itself; the library is never
// built that way, and its kernel arguments are the same in either build.
#ifdef KVP_TIMING
__device__ unsigned long long *kvp_timing_stamps;  // [item][32]
__device__ unsigned long long *kvp_timing_phases;  // [item][8 waves][8]
#define KVP_STAMP(slot) do { if (threadIdx.x == 0 && (slot) < 32 && kvp_timing_stamps) kvp_timing_stamps[blockIdx.x * 32 + (slot)] = wall_clock64(); } while (0)
// per-wave cycle totals of the tile loop's phases
#define KVP_PHASE_DECL unsigned long long ph_acc[6] = {0, 0, 0, 0, 0, 0}, ph_last = __builtin_readcyclecounter()
#define KVP_PHASE(i) do { const unsigned long long t_ = __builtin_readcyclecounter(); ph_acc[i] += t_ - ph_last; ph_last = t_; } while (0)
#define KVP_PHASE_WRITE do { if ((threadIdx.x & 63) == 0 && kvp_timing_phases) for (int i_ = 0; i_ < 6; ++i_) kvp_timing_phases[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 8 + i_] = ph_acc[i_]; } while (0)
#else
#define KVP_STAMP(slot) do {} while (0)
#define KVP_PHASE_DECL do {} while (0)
#define KVP_PHASE(i) do {} while (0)
#define KVP_PHASE_WRITE do {} while (0)
#endif

// The query is held rotated and multiplied by log2(e)/sqrt(d), so S = K Q^T is in log2
// units.  The S accumulators start at -m_ref: after the MFMAs they hold s - m_ref and the
// probabilities are exp2 of them with no further arithmetic.
//
// SRC_CONTIG / SRC_PAGED: an item's [kv_begin, kv_end) are cache rows.
// SRC_PACKETS: no cache exists; [kv_begin, kv_end) index a.tiles, each tile up to 64 rows of
// one stored packet (read in place from the arena) or of the query rows (rotated K_new in
// a.k_tail, V_new as given).  The keys of a stored packet stay at their local positions;
// instead the query is rotated by (ctx_len + t) - Delta_j for that packet's tiles, which
// gives the same scores (Eq. 1: scores depend on the position difference only).
//
// NW wavefronts per workgroup in KS groups of RW = NW / KS; a wave owns 32 packed rows, a
// group owns BM = 32 RW rows, and all NW waves share the loading of every K/V tile.
//   NW 4, KS 1, 2 stages: two workgroups share a CU (small row blocks, many items);
//   NW 8, KS 1, 4 stages: each K/V row is fetched once per 256 packed rows, three tiles in
//                         flight, one workgroup per CU;
//   NW 8, KS 2, 4 stages: 128 rows, the two groups take alternate tiles of the item's range
//                         (an in-workgroup split-KV that halves the serial chain of a
//                         latency-bound item) and merge their (m, l, O) through LDS.
template <int STAGES, int SRC, int NW, int KS, bool NTL>
__device__ __forceinline__ void attention_body(const AttnArgs &a)
{
    constexpr int RW = NW / KS;    // waves per group (a group owns 32 RW rows)
    constexpr int NT = 64 * NW;    // threads
    constexpr int NI = 16 / NW;    // K (and V) load instructions per wave per tile
    constexpr int PR = STAGES / KS - 1;  // rounds (of KS tiles) loaded ahead
    static_assert(STAGES % KS == 0 && PR >= 1, "stages");
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    KVP_STAMP(0);
    const AttnItem it = a.inl.n ? attn_inline_item(a.inl, blockIdx.x, a.n_kv, a.part_stride) : a.items[blockIdx.x];
    if (it.n_rows <= 0) return;  // padding item of the launch order
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_r = wave % RW, grp = wave / RW;  // row wave inside its group, group
    const int n = lane & 31, h = lane >> 5;
    const int g = a.g;

    const bf16_t *kc = (const bf16_t *)a.cache.k;
    const bf16_t *vc = (const bf16_t *)a.cache.v;
    const int kv_last = it.kv_end - 1;
    const int n_tiles = SRC == SRC_PACKETS ? it.kv_end - it.kv_begin : (it.kv_end - it.kv_begin + BN - 1) / BN;

    // paged layout: this item's block ids go to LDS once, so the tile loop issues no
    // ordinary global loads (its in-flight count is what the waits below rely on)
    int *blk_ids = (int *)(lds + STAGES * STAGE_BYTES);
    const int blk0 = SRC == SRC_PAGED ? (it.kv_begin >> a.cache.block_shift) : 0;
    // contiguous layout: wave-uniform byte address of the item's first K / V row
    const int64_t contig_off = SRC == SRC_CONTIG
                                   ? (int64_t)it.req * a.cache.req_stride + (int64_t)a.layer * a.cache.layer_stride +
                                         ((int64_t)it.kv_head * a.cache.t_cap + it.kv_begin) * D
                                   : 0;
    const char *k_item = (const char *)(kc + contig_off);
    const char *v_item = (const char *)(vc + contig_off);
    const int64_t paged_base = (int64_t)a.layer * a.cache.layer_stride;
    // packets: rows of the query's own K (rotated, in a.k_tail) and V (a.v_new) for this head
    const int64_t tail_off = ((int64_t)it.q_off * a.n_kv + it.kv_head) * D;

    // direct HBM -> LDS load of tile tj: wave w, instruction i fills tile rows
    // 4 (NW i + w) .. +3 (1 KiB contiguous in LDS); lane l owns slot (row + l / 16, chunk l % 16)
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds);
    const int slot_row = lane >> 4, slot_chunk = lane & 15;
    const int k_chunk = slot_chunk ^ ((4 * wave + slot_row) & 15);  // logical chunk fetched
    const int v_chunk = slot_chunk ^ (4 * slot_row);
    const int last_tile_rows = it.kv_end - it.kv_begin - (n_tiles - 1) * BN;  // 1..64 (cache modes)
    // paged layout: the LDS word with the block id of load instruction i of tile tj.  The 4 rows
    // of one instruction lie in one block (blocks hold a multiple of 4 rows, items start at a
    // multiple of 64), clamped rows included, so the word is the same for the whole wave.
    auto blk_word = [&](int tj, int i) -> int {
        const int max_r = tj == n_tiles - 1 ? last_tile_rows - 1 : BN - 1;
        const int rb = 4 * (NW * i + wave) < max_r ? 4 * (NW * i + wave) : max_r;
        return blk_ids[((it.kv_begin + tj * BN + rb) >> a.cache.block_shift) - blk0];
    };
    // The loads of tile tj: NI parts per wave, each one K and one V load instruction.  tile_src
    // is the scalar part (where the tile's rows are), issue_part the per-lane part.
    struct TileSrc {
        const char *kt, *vt;   // wave-uniform byte address of the tile's first K / V row
        uint32_t row_bytes;    // distance between rows
        int max_r;             // last row of the tile that exists (rows past it repeat it; they are masked later)
    };
    auto tile_src = [&](int tj) -> TileSrc {
        TileSrc ts;
        if (SRC == SRC_PACKETS) {
            const AttnTile td = load_tile_record(a.tiles, it.kv_begin + tj);
            if (td.kind == 0) {
                // stride < 0: a compressed packet, src_base is this layer's own part of the blob
                // ([K: Hkv x rows][V: Hkv x rows], rows = -stride)
                const bool own_layer = td.stride < 0;
                const int stride = own_layer ? -td.stride : td.stride;
                const int64_t slice = ((int64_t)(own_layer ? 0 : a.layer) * a.n_kv + it.kv_head) * stride + td.row0;
                ts.kt = (const char *)((const bf16_t *)a.arena + td.src_base + slice * D);
                ts.vt = ts.kt + (int64_t)(own_layer ? 1 : a.n_layers_total) * a.n_kv * stride * ROW_BYTES;
                ts.row_bytes = ROW_BYTES;
            } else {
                ts.kt = (const char *)((const bf16_t *)a.k_tail + tail_off + (int64_t)td.row0 * a.n_kv * D);
                ts.vt = (const char *)((const bf16_t *)a.v_new + tail_off + (int64_t)td.row0 * a.n_kv * D);
                ts.row_bytes = (uint32_t)(a.n_kv * ROW_BYTES);
            }
            ts.kt = uniform_ptr(ts.kt);
            ts.vt = uniform_ptr(ts.vt);
            ts.max_r = td.n_rows - 1;
            return ts;
        }
        ts.max_r = tj == n_tiles - 1 ? last_tile_rows - 1 : BN - 1;
        ts.row_bytes = ROW_BYTES;
        if (SRC == SRC_CONTIG) {
            ts.kt = uniform_ptr(k_item + (int64_t)tj * TILE_BYTES);
            ts.vt = uniform_ptr(v_item + (int64_t)tj * TILE_BYTES);
        } else {
            ts.kt = ts.vt = nullptr;  // (paged: every load instruction looks its block up)
        }
        return ts;
    };
    auto issue_part = [&](const TileSrc &ts, int tj, int i) {
        const uint32_t st = lds_base + (uint32_t)((tj % STAGES) * STAGE_BYTES);
        int r = 4 * (NW * i + wave) + slot_row;
        r = r < ts.max_r ? r : ts.max_r;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(st + (uint32_t)(4 * (NW * i + wave) * ROW_BYTES));  // (wave-uniform)
        if (SRC != SRC_PAGED) {
            // (uniform_ptr again: should the compiler have moved the address to vector registers, it
            // comes back to scalar ones, which the instruction needs; otherwise this folds away)
            load_to_lds_16<NTL>(uniform_ptr(ts.kt), (uint32_t)r * ts.row_bytes + 16 * k_chunk, dst);
            load_to_lds_16<NTL>(uniform_ptr(ts.vt), (uint32_t)r * ts.row_bytes + 16 * v_chunk, dst + TILE_BYTES);
        } else {
            // the block id is wave-uniform: the address is a scalar base plus a 32-bit lane offset
            const int b = __builtin_amdgcn_readfirstlane(blk_word(tj, i));
            const int64_t blk_off = paged_base + (((int64_t)b * a.n_kv + it.kv_head) << a.cache.block_shift) * D;
            const int slot = (it.kv_begin + tj * BN + r) & ((1 << a.cache.block_shift) - 1);
            const char *kt = uniform_ptr((const char *)(kc + blk_off));
            const char *vt = uniform_ptr((const char *)(vc + blk_off));
            load_to_lds_16<NTL>(kt, (uint32_t)(slot * ROW_BYTES + 16 * k_chunk), dst);
            load_to_lds_16<NTL>(vt, (uint32_t)(slot * ROW_BYTES + 16 * v_chunk), dst + TILE_BYTES);
        }
    };
    auto issue = [&](int tj) {
        const TileSrc ts = tile_src(tj);
#pragma unroll
        for (int i = 0; i < NI; ++i) issue_part(ts, tj, i);
    };
    // this lane's query row
    const int rr = 32 * wave_r + n;
    const bool row_ok = rr < it.n_rows;
    const bool wave_active = 32 * wave_r < it.n_rows;  // wave-uniform
    const int m = it.m0 + (row_ok ? rr : 0);
    const int t = m / g, hq = it.kv_head * g + m % g;
    const int limit = row_ok ? it.ctx_len + t + 1 : 0;  // cache modes: kv rows [0, limit) are visible
    // smallest limit among the wave's rows (rows are ordered by query token)
    const int wave_limit = it.ctx_len + (it.m0 + 32 * wave_r) / g + 1;

    // B operand of S^T = K Q^T: lane holds Q[m][16 ks + 8 h .. +7] for ks = 0..7, rotated by
    // `rel` positions and multiplied by log2(e)/sqrt(d).  Element 16 ks + 8 h + j (ks < 4)
    // pairs with the same slot of ks + 4, so the rotation stays inside the lane.
    bf16x8 qf[8];
    const bf16_t *qp = (const bf16_t *)a.q + ((int64_t)(it.q_off + t) * a.n_q_heads + hq) * D + 8 * h;
    const int q_pos = a.prerotated ? 0 : it.pos0 + t;  // rotation the query still needs
    u32x4_t qraw[8], csraw[16];
    auto q_issue = [&](int delta) {  // 24 loads: the raw query row and the (cos, sin) of its rotation
        const bf16_t *qsrc = row_ok ? qp : (const bf16_t *)a.q + 8 * h;  // idle lanes read row 0 (and drop it)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qraw[ks] = load16_nowait(qsrc + 16 * ks);
        const int rel = row_ok ? q_pos - delta : 0;
        const float4 *csr = (const float4 *)(a.cs + (int64_t)(rel < 0 ? -rel : rel) * 64 + 8 * h);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int j = 0; j < 4; ++j) csraw[4 * ks + j] = load16_nowait(csr + 8 * ks + j);
    };
    // `younger`: tiles whose loads were issued after q_issue and may still be on their way
    auto q_finish = [&](int delta, int younger) {
        if (younger >= 3) wait_vmcnt<3 * 2 * NI>();
        else if (younger == 2) wait_vmcnt<2 * 2 * NI>();
        else if (younger == 1) wait_vmcnt<2 * NI>();
        else wait_vmcnt<0>();
        // the registers are valid from here on: keep every use below this point
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(qraw[i]));
#pragma unroll
        for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(csraw[i]));
        const int rel = row_ok ? q_pos - delta : 0;
        const float sign = rel < 0 ? -1.f : 1.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            float4 cs4[4];  // (cos, sin) pairs of elements 16 ks + 8 h + 2 j, + 1
#pragma unroll
            for (int j = 0; j < 4; ++j) cs4[j] = __builtin_bit_cast(float4, csraw[4 * ks + j]);
            uint4 lo = __builtin_bit_cast(uint4, qraw[ks]), hi = __builtin_bit_cast(uint4, qraw[ks + 4]);
            if (!row_ok) lo = hi = make_uint4(0, 0, 0, 0);
            uint4 olo, ohi;
            rotate_chunk_pair<false>(lo, hi, cs4, sign, a.scale_log2e, olo, ohi);
            qf[ks] = __builtin_bit_cast(bf16x8, olo);
            qf[ks + 4] = __builtin_bit_cast(bf16x8, ohi);
        }
        // pinned: nothing of this is recomputed or waited for inside the tile loop
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks]));
    };
    // Re-rotation inside the tile loop (in-place packet reads, at every packet boundary): plain
    // loads, whose wait the compiler places (it drains the tile loads in flight as well).
    auto reload_q = [&](int delta) {
        uint4 qr[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qr[ks] = row_ok ? *(const uint4 *)(qp + 16 * ks) : make_uint4(0, 0, 0, 0);
        const int rel = row_ok ? q_pos - delta : 0;
        const float sign = rel < 0 ? -1.f : 1.f;
        const float4 *csr = (const float4 *)(a.cs + (int64_t)(rel < 0 ? -rel : rel) * 64 + 8 * h);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            float4 cs4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) cs4[j] = csr[8 * ks + j];
            uint4 olo, ohi;
            rotate_chunk_pair<false>(qr[ks], qr[ks + 4], cs4, sign, a.scale_log2e, olo, ohi);
            qf[ks] = __builtin_bit_cast(bf16x8, olo);
            qf[ks + 4] = __builtin_bit_cast(bf16x8, ohi);
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks]));
    };
    int cur_delta = SRC == SRC_PACKETS && n_tiles > 0 ? load_tile_record(a.tiles, it.kv_begin).pos : 0;
    KVP_STAMP(1);
    q_issue(cur_delta);  // first, so that the query arrives ahead of the tiles
    if (SRC == SRC_PAGED) {  // the block ids travel while the query does
        const int nb = (kv_last >> a.cache.block_shift) - blk0 + 1;
        for (int i = tid; i < nb; i += NT)
            blk_ids[i] = a.cache.block_table[(int64_t)it.req * a.cache.max_blocks + blk0 + i];
        __syncthreads();
    }
    // a first tile that cannot contain query rows can start its trip right away
    const bool early0 = n_tiles > 0 && (SRC == SRC_PACKETS ? load_tile_record(a.tiles, it.kv_begin).kind == 0 : it.kv_begin + BN <= it.ctx_len);
    if (early0) issue(0);

    // ---- query rows inside this item's range: rotate K_new to its row's position and
    // append K_new / V_new before any tile load can touch those rows
    {
        int tail_lo, n_tail;  // query rows [tail_lo, tail_lo + n_tail) relative to ctx_len
        if (SRC == SRC_PACKETS) {
            // an item that reaches the query tiles writes all of this head's rotated K_new rows
            const bool has_tail = n_tiles > 0 && load_tile_record(a.tiles, it.kv_end - 1).kind != 0;
            tail_lo = 0;
            n_tail = has_tail ? it.n_q : 0;
        } else {
            tail_lo = (it.kv_begin > it.ctx_len ? it.kv_begin : it.ctx_len) - it.ctx_len;
            n_tail = it.kv_end - it.ctx_len - tail_lo;  // > 0 only for items that reach the query rows
        }
        if (n_tail > 0) {
            bf16_t *kcw = SRC == SRC_PACKETS ? (bf16_t *)a.k_tail : (bf16_t *)a.cache.k;
            bf16_t *vcw = (bf16_t *)a.cache.v;
            // Work units: 8 K chunk pairs per row (rotate, store) and, with a cache, 16 V chunks per
            // row (copy).  A thread takes two K units and four V units per trip and issues all their
            // loads before it uses the first, so the append costs one memory round trip per trip
            // (32 query rows: one trip) instead of one per unit.
            auto unit_dst = [&](int qr, int64_t src) -> int64_t {
                const int row = it.ctx_len + qr;  // cache row of the query token
                if (SRC == SRC_PACKETS) return src;
                if (SRC == SRC_CONTIG) return contig_off + (int64_t)(row - it.kv_begin) * D;
                const int b = blk_ids[(row >> a.cache.block_shift) - blk0];
                const int slot = row & ((1 << a.cache.block_shift) - 1);
                return paged_base + ((((int64_t)b * a.n_kv + it.kv_head) << a.cache.block_shift) + slot) * D;
            };
            const int n_k = n_tail * 8, n_v = SRC == SRC_PACKETS ? 0 : n_tail * 16;
            // (loads are unconditional, from units clamped into range; only the stores are guarded)
            for (int s0 = 0; 2 * s0 * NT < n_k || 4 * s0 * NT < n_v; ++s0) {
                if (4 * s0 * NT + tid >= n_v && 2 * s0 * NT + tid >= n_k) continue;  // (a thread without a unit: few query rows)
                uint4 vv0, vv1, vv2, vv3;
                int64_t vd0, vd1, vd2, vd3;
                auto v_load = [&](int j, uint4 &vv, int64_t &vd) -> bool {
                    const int idx = (4 * s0 + j) * NT + tid;
                    const int ic = idx < n_v ? idx : (n_v > 0 ? n_v - 1 : 0);
                    const int qr = tail_lo + ic / 16, e = 8 * (ic % 16);
                    const int64_t src = ((int64_t)(it.q_off + qr) * a.n_kv + it.kv_head) * D;
                    vd = unit_dst(qr, src) + e;
                    vv = n_v > 0 ? *(const uint4 *)((const bf16_t *)a.v_new + src + e) : make_uint4(0, 0, 0, 0);
                    return idx < n_v;
                };
                const bool von0 = v_load(0, vv0, vd0), von1 = v_load(1, vv1, vd1), von2 = v_load(2, vv2, vd2), von3 = v_load(3, vv3, vd3);
                struct KUnit { uint4 ulo, uhi; float4 c0, c1, c2, c3; int64_t dst; bool on; };
                auto k_load = [&](int j) -> KUnit {
                    KUnit u;
                    const int idx = (2 * s0 + j) * NT + tid;
                    const int ic = idx < n_k ? idx : n_k - 1;
                    const int qr = tail_lo + ic / 8, e = 8 * (ic % 8);
                    const int pos = it.pos0 + qr;     // the token's position
                    const int64_t src = ((int64_t)(it.q_off + qr) * a.n_kv + it.kv_head) * D;
                    u.dst = unit_dst(qr, src) + e;
                    u.ulo = *(const uint4 *)((const bf16_t *)a.k_new + src + e);
                    u.uhi = *(const uint4 *)((const bf16_t *)a.k_new + src + 64 + e);
                    const float4 *csr = (const float4 *)(a.cs + (int64_t)pos * 64 + e);
                    u.c0 = csr[0]; u.c1 = csr[1]; u.c2 = csr[2]; u.c3 = csr[3];
                    u.on = idx < n_k;
                    return u;
                };
                const KUnit k0 = k_load(0), k1 = k_load(1);
                if (von0) *(uint4 *)(vcw + vd0) = vv0;
                if (von1) *(uint4 *)(vcw + vd1) = vv1;
                if (von2) *(uint4 *)(vcw + vd2) = vv2;
                if (von3) *(uint4 *)(vcw + vd3) = vv3;
                auto k_store = [&](const KUnit &u) {
                    if (!u.on) return;
                    const float4 one = make_float4(1.f, 0.f, 1.f, 0.f);
                    const float4 cs4[4] = {a.prerotated ? one : u.c0, a.prerotated ? one : u.c1, a.prerotated ? one : u.c2, a.prerotated ? one : u.c3};
                    uint4 olo, ohi;
                    rotate_chunk_pair<true>(u.ulo, u.uhi, cs4, 1.f, 1.f, olo, ohi);
                    *(uint4 *)(kcw + u.dst) = olo;
                    *(uint4 *)(kcw + u.dst + 64) = ohi;
                };
                k_store(k0);
                k_store(k1);
            }
            wait_vmcnt<0>();   // this wave's stores have reached the L2
            // The same wait once more, in the form the compiler's own wait bookkeeping understands:
            // without it the compiler takes the loads and stores above for still outstanding when the
            // tile loop is entered and puts a full vmcnt(0) in front of every tile's first MFMA -- which
            // waits for every tile load in flight and turns a four-stage ring into a one-deep prefetch.
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), the other counters left alone
            __syncthreads();   // ... and so have every other wave's
        }
    }

#pragma unroll
    for (int s = 0; s < KS * PR; ++s)
        if (s < n_tiles && !(s == 0 && early0)) issue(s);

    q_finish(cur_delta, n_tiles < KS * PR ? n_tiles : KS * PR);
    KVP_STAMP(2);

    floatx16 oacc[4];
#pragma unroll
    for (int eb = 0; eb < 4; ++eb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[eb][r] = 0.f;
    float m_ref = -INFINITY, l_i = 0.f;  // reference max (log2 units) and running sum
    // -m_ref in all 16 slots (every accumulator of a lane belongs to the same query row): the
    // first S MFMA of a tile takes it as its C operand, so S - m_ref costs no extra instruction.
    // Rewritten only when the reference moves; pinned so that it is not rebuilt per tile.
    // (The in-place packet variant has no registers to spare and rebuilds it per tile.)
    constexpr bool KEEP_CINIT = SRC != SRC_PACKETS;
    floatx16 cinit;
#pragma unroll
    for (int r = 0; r < 16; ++r) cinit[r] = 0.f;
    if (KEEP_CINIT) asm volatile("" : "+v"(cinit));

    const int tr_row = (lane & 15) >> 2;
    const int tr_x = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);  // 16-byte chunk inside the 64-byte column group
    const int tr_half = 8 * (lane & 1);


    const int n_rounds = (n_tiles + KS - 1) / KS;
    KVP_PHASE_DECL;
    for (int rd = 0; rd < n_rounds; ++rd) {
        KVP_PHASE(5);
        // round rd's tiles have landed once only the loads of the rounds issued after it remain
        {
            const int hi = KS * (rd + PR) < n_tiles ? KS * (rd + PR) : n_tiles;
            const int lo = KS * (rd + 1) < n_tiles ? KS * (rd + 1) : n_tiles;
            const int younger = hi - lo;  // tiles issued after this round, 0 .. KS (PR - 1)
            if (younger >= 3) wait_vmcnt<3 * 2 * NI>();
            else if (younger == 2) wait_vmcnt<2 * 2 * NI>();
            else if (younger == 1) wait_vmcnt<2 * NI>();
            else wait_vmcnt<0>();
        }
        KVP_STAMP(4 + 2 * rd);
        KVP_PHASE(0);
        wg_barrier();  // every wave's part of the round is in LDS; everyone is done with round rd-1
        KVP_STAMP(5 + 2 * rd);
        KVP_PHASE(1);
        auto refill = [&]() {  // the stages round rd-1 used take round rd+PR
#pragma unroll
            for (int k2 = 0; k2 < KS; ++k2)
                if (KS * (rd + PR) + k2 < n_tiles) issue(KS * (rd + PR) + k2);
        };
        const int ti = KS * rd + grp;  // this group's tile of the round
        if (ti >= n_tiles || !wave_active) {  // nothing to compute: only help to load
            refill();
            continue;
        }

        const int kv0 = it.kv_begin + ti * BN;
        const char *kl = lds + (ti % STAGES) * STAGE_BYTES;
        const char *vl = kl + TILE_BYTES;
        AttnTile td;
        if (SRC == SRC_PACKETS) {
            td = load_tile_record(a.tiles, it.kv_begin + ti);
            if (td.pos != cur_delta && wave_active) {  // the tile belongs to another packet: re-rotate the query
                cur_delta = td.pos;
                reload_q(cur_delta);
            }
        }

        // ---- S^T - m_ref = K Q^T - m_ref : 2 blocks of 32 kv rows x 32 query rows
        floatx16 sacc[2];
        if (!KEEP_CINIT) {
            const float c = m_ref == -INFINITY ? 0.f : -m_ref;
#pragma unroll
            for (int r = 0; r < 16; ++r) cinit[r] = c;
        }
        // K fragments run AHEAD k-steps in front of the MFMAs that use them: the first AHEAD k-steps'
        // fragments are requested up front, and each k-step's MFMA pair is followed by the request
        // for the fragments AHEAD steps on, so the matrix pipe starts after a quarter of the tile has
        // arrived from LDS instead of all of it (the four waves of a workgroup reach this point
        // together, and 64 KB of fragment reads keep the LDS busy for about as long as the 16 MFMAs
        // keep the matrix pipe).
        // The next tile loads -- they refill the stages the previous round used, which every wave
        // left before the barrier above -- are issued between the matrix instructions too, one part
        // (a K and a V load with their address arithmetic) behind each of the first k-steps' MFMA
        // pair: the matrix pipe is busy for 64 cycles per pair, about what a part takes to issue.
        {
            constexpr int AHEAD = 2;  // (2, 3, 4, 6 and 8 k-steps measured: 2 is the fastest by a little, and holds the fewest registers)
            constexpr int N_PARTS = KS * NI;                   // <= 4
            static_assert(N_PARTS <= 8, "one part per k-step");
            TileSrc rsrc[KS];
#pragma unroll
            for (int k2 = 0; k2 < KS; ++k2)
                if (KS * (rd + PR) + k2 < n_tiles) rsrc[k2] = tile_src(KS * (rd + PR) + k2);
            uint4 kf[2 * AHEAD];
            auto read_k = [&](int kstep) {
                const int coff = 16 * ((2 * kstep + h) ^ (n & 15));
                kf[2 * (kstep % AHEAD)] = *(const uint4 *)(kl + n * ROW_BYTES + coff);
                kf[2 * (kstep % AHEAD) + 1] = *(const uint4 *)(kl + (32 + n) * ROW_BYTES + coff);
            };
#pragma unroll
            for (int i = 0; i < AHEAD; ++i) read_k(i);
            __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the matrix code
#pragma unroll
            for (int kstep = 0; kstep < 8; ++kstep) {
                const bool head = kstep == 0;  // compile-time: the tile's first k-step
                const int sl = 2 * (kstep % AHEAD);
                sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[sl]), qf[kstep], head ? cinit : sacc[0], 0, 0, 0);
                sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[sl + 1]), qf[kstep], head ? cinit : sacc[1], 0, 0, 0);
                if (kstep + AHEAD < 8) read_k(kstep + AHEAD);
                if (kstep < N_PARTS) {
                    const int k2 = kstep / NI, tj = KS * (rd + PR) + k2;
                    if (tj < n_tiles) issue_part(rsrc[k2], tj, kstep % NI);
                }
                __builtin_amdgcn_sched_barrier(0);  // what follows a pair stays behind it
            }
        }
        KVP_PHASE(2);

        // ---- online softmax; accumulator r of block kb is tile row 32 kb + 8 (r/4) + 4 h + r%4
        if (SRC == SRC_PACKETS) {
            if (td.kind != 0 || td.n_rows < BN) {  // wave-uniform: query tiles and ragged packet ends
                const int vis = td.kind != 0 ? (row_ok ? t - td.row0 + 1 : 0) : BN;  // causal among query rows
                const int lim = vis < td.n_rows ? vis : td.n_rows;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * kb + 8 * (r >> 2) + 4 * h + (r & 3) >= lim) sacc[kb][r] = -INFINITY;
            }
        } else if (kv0 + BN > wave_limit || kv0 + BN > it.kv_end) {  // wave-uniform: tail tiles only
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int kv = kv0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (kv >= limit || kv >= it.kv_end) sacc[kb][r] = -INFINITY;
                }
        }
        float mx = max3(sacc[0][0], sacc[1][0], sacc[0][1]);
        mx = max3(mx, sacc[1][1], sacc[0][2]);
#pragma unroll
        for (int r = 2; r < 15; ++r) mx = max3(mx, sacc[1][r], sacc[0][r + 1]);
        mx = fmaxf(mx, sacc[1][15]);
        mx = xhalf_max(mx);  // row max relative to m_ref
        // The reference moves when a row sees its first visible entry (it becomes that
        // tile's maximum) and afterwards only when the maximum outgrows the slack.
        const bool first = m_ref == -INFINITY;
        const bool move = first ? mx > -INFINITY : mx > RESCALE_SLACK;
        if (__any(move)) {  // wave-uniform; rare once the maxima settle
            const float delta = move ? mx : 0.f;
            const float alpha = first ? 1.f : __builtin_amdgcn_exp2f(-delta);  // first: O = l = 0
            m_ref = first ? (move ? mx : -INFINITY) : m_ref + delta;
            l_i *= alpha;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[kb][r] -= delta;
#pragma unroll
            for (int eb = 0; eb < 4; ++eb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[eb][r] *= alpha;
            if (KEEP_CINIT) {
                const float c = m_ref == -INFINITY ? 0.f : -m_ref;
#pragma unroll
                for (int r = 0; r < 16; ++r) cinit[r] = c;
                asm volatile("" : "+v"(cinit));
            }
        }

        // ---- P = exp2(S - m_ref) and O^T += V^T P^T, one 32-row block at a time so that the
        // exponentials of block 1 run while the matrix cores accumulate block 0.
        // k-step j of block kb covers tile rows 32 kb + 16 j + [0, 16); P^T slots 0..7 of
        // lane-half h are rows 4h+{0..3} and 8+4h+{0..3} of that step, so the two transposing
        // reads fetch exactly those rows of V for column 32 eb + n.
        KVP_PHASE(3);
        float rs0 = 0.f, rs1 = 0.f;
        const bf16x2 bf16_ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
        typedef __attribute__((address_space(3))) short4v *lds_s4;
        short4v vfr[2][8];  // V fragments of one k-step: [buffer][2 eb + lo/hi]
        auto read_v = [&](int step, int buf) {  // step = 2 kb + j
            const char *vp = vl + (16 * step + 4 * h + tr_row) * ROW_BYTES + tr_half;
#pragma unroll
            for (int eb = 0; eb < 4; ++eb) {
                const int coff = 16 * (4 * (eb ^ tr_row) + tr_x);
                vfr[buf][2 * eb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(vp + coff));
                vfr[buf][2 * eb + 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(vp + 8 * ROW_BYTES + coff));
            }
        };
        read_v(0, 0);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            uint32_t pk[8];
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                float p0 = __builtin_amdgcn_exp2f(sacc[kb][r]);
                float p1 = __builtin_amdgcn_exp2f(sacc[kb][r + 1]);
                pk[r >> 1] = pack_bf16_hw(p0, p1);
                // the row sum takes the rounded values, i.e. exactly what multiplies V
                const bf16x2 pp = __builtin_bit_cast(bf16x2, pk[r >> 1]);
                if (r & 2) rs1 = __builtin_amdgcn_fdot2_f32_bf16(pp, bf16_ones, rs1, false);
                else rs0 = __builtin_amdgcn_fdot2_f32_bf16(pp, bf16_ones, rs0, false);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int step = 2 * kb + j;
                if (step + 1 < 4) read_v(step + 1, (step + 1) & 1);  // next k-step's V lands under these MFMAs
                uint4 pu = make_uint4(pk[4 * j], pk[4 * j + 1], pk[4 * j + 2], pk[4 * j + 3]);
                bf16x8 pf = __builtin_bit_cast(bf16x8, pu);
#pragma unroll
                for (int eb = 0; eb < 4; ++eb) {
                    union { short4v s[2]; bf16x8 v; } vf;
                    vf.s[0] = vfr[step & 1][2 * eb];
                    vf.s[1] = vfr[step & 1][2 * eb + 1];
                    oacc[eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf, oacc[eb], 0, 0, 0);
                }
            }
        }
        l_i += rs0 + rs1;  // this lane's half of the row; the halves are added once, at the end
        KVP_PHASE(4);
    }
    KVP_PHASE_WRITE;
    l_i = xhalf_sum(l_i);
    KVP_STAMP(30);

    if (KS == 2) {
        // ---- merge the two groups' (m, l, O) of each row through LDS (the tile stages are free
        // once every wave has left the loop): group 1 writes, group 0 folds it in and goes on.
        wg_barrier();
        float *xo = (float *)lds;                      // [16][RW][64 lanes][4]
        float *xm = xo + 16 * RW * 64 * 4;             // [RW][64] m, then [RW][64] l
        if (grp == 1) {
#pragma unroll
            for (int eb = 0; eb < 4; ++eb)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *(float4 *)(xo + (((4 * eb + q4) * RW + wave_r) * 64 + lane) * 4) =
                        make_float4(oacc[eb][4 * q4], oacc[eb][4 * q4 + 1], oacc[eb][4 * q4 + 2], oacc[eb][4 * q4 + 3]);
            xm[wave_r * 64 + lane] = m_ref;
            xm[RW * 64 + wave_r * 64 + lane] = l_i;
        }
        __syncthreads();
        if (grp == 1) return;
        const float m1 = xm[wave_r * 64 + lane], l1 = xm[RW * 64 + wave_r * 64 + lane];
        const float mm = fmaxf(m_ref, m1);
        const float a0 = m_ref == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_ref - mm);
        const float a1 = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m1 - mm);
        m_ref = mm;
        l_i = l_i * a0 + l1 * a1;
#pragma unroll
        for (int eb = 0; eb < 4; ++eb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float4 o1 = *(const float4 *)(xo + (((4 * eb + q4) * RW + wave_r) * 64 + lane) * 4);
                oacc[eb][4 * q4] = oacc[eb][4 * q4] * a0 + o1.x * a1;
                oacc[eb][4 * q4 + 1] = oacc[eb][4 * q4 + 1] * a0 + o1.y * a1;
                oacc[eb][4 * q4 + 2] = oacc[eb][4 * q4 + 2] * a0 + o1.z * a1;
                oacc[eb][4 * q4 + 3] = oacc[eb][4 * q4 + 3] * a0 + o1.w * a1;
            }
    }

    // ---- epilogue: lane holds O[m][32 eb + 8 (r/4) + 4 h + r%4]
    if (row_ok) {
        if (it.part_slot < 0) {
            bf16_t *op = (bf16_t *)a.out + ((int64_t)(it.q_off + t) * a.n_q_heads + hq) * D;
            const float inv = 1.f / l_i;
#pragma unroll
            for (int eb = 0; eb < 4; ++eb)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    uint2 u;
                    u.x = pack_bf16_hw(oacc[eb][4 * q4] * inv, oacc[eb][4 * q4 + 1] * inv);
                    u.y = pack_bf16_hw(oacc[eb][4 * q4 + 2] * inv, oacc[eb][4 * q4 + 3] * inv);
                    *(uint2 *)(op + 32 * eb + 8 * q4 + 4 * h) = u;
                }
        }
    }
    if (it.part_slot >= 0) {
        // A slot holds a.bm rows of D fp16 values (the launch's largest row block; BM <= a.bm), then
        // m and l of each row in fp32.  A row of the split's unnormalised O goes out as fp16 scaled
        // by a power of two 2^-e that brings its largest magnitude below 1; m + e and l 2^-e go with
        // it, which is the same partial result relative to another reference, so the merge's
        // algebra does not change.  Eleven significant bits relative to the row's maximum, where the
        // bf16 output keeps eight.
        char *pp = (char *)a.partials + (int64_t)it.part_slot * part_slot_bytes(a.bm, D, 1);
        float amax = 0.f;
#pragma unroll
        for (int eb = 0; eb < 4; ++eb)
#pragma unroll
            for (int r = 0; r < 16; ++r) amax = fmaxf(amax, __builtin_fabsf(oacc[eb][r]));
        amax = xhalf_max(amax);
        int e = amax > 0.f ? __builtin_amdgcn_frexp_expf(amax) : 0;  // amax = f 2^e with f in [0.5, 1)
        e = e < -100 ? -100 : (e > 120 ? 120 : e);                   // (keeps l 2^-e and 2^-e itself in range)
        const float sc = __builtin_ldexpf(1.f, -e);
        typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
        auto pack4 = [&](int eb, int q4) -> uint2 {  // four neighbouring columns of this lane's row
            const floatx2 lo = {oacc[eb][4 * q4] * sc, oacc[eb][4 * q4 + 1] * sc};
            const floatx2 hi = {oacc[eb][4 * q4 + 2] * sc, oacc[eb][4 * q4 + 3] * sc};
            return make_uint2(__builtin_bit_cast(uint32_t, __builtin_convertvector(lo, halfx2)),
                              __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, halfx2)));
        };
        // The rows go through LDS so that they leave as whole 256-byte rows (four per store
        // instruction) instead of 16-byte pieces: each wave parks its 32 x 128 halves in 8 KiB of its
        // own in the (now idle) tile stages, 8-byte chunk c of row n at chunk c ^ n, and reads them
        // back row by row.  (KS = 2: the merge above has used the first 66 KiB; the rows go behind.)
        if (KS == 1) wg_barrier();  // every wave is done with the tiles
        char *reg = lds + (KS == 2 ? 68 * 1024 : 0) + wave_r * (32 * D * 2);
#pragma unroll
        for (int eb = 0; eb < 4; ++eb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) *(uint2 *)(reg + n * (D * 2) + 8 * ((8 * eb + 2 * q4 + h) ^ n)) = pack4(eb, q4);
        // (a wave reads only what it wrote itself: no barrier, the compiler orders the two)
        const int c = lane & 15;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = 4 * j + (lane >> 4);
            // logical 8-byte chunks 2c and 2c + 1 of row r sit in the 16-byte unit c ^ (r >> 1), swapped when r is odd
            uint4 f = *(const uint4 *)(reg + r * (D * 2) + 16 * (c ^ (r >> 1)));
            if (r & 1) f = make_uint4(f.z, f.w, f.x, f.y);
            if (32 * wave_r + r < it.n_rows) *(uint4 *)(pp + (int64_t)(32 * wave_r + r) * (D * 2) + 16 * c) = f;
        }
        if (row_ok && h == 0) {
            float *ml = (float *)(pp + part_rows_bytes(a.bm, D, 1));
            ml[rr] = m_ref == -INFINITY ? -INFINITY : m_ref + (float)e;
            ml[a.bm + rr] = l_i * sc;
        }
    }
    KVP_STAMP(31);
}

template <int STAGES, int SRC, int NW, int KS, bool NTL>
__global__ __launch_bounds__(64 * NW, 2) void attention_mfma_kernel(AttnArgs a)
{
    attention_body<STAGES, SRC, NW, KS, NTL>(a);
}

// 8 waves, 4 stages, the row block chosen item by item: 256 packed rows, or (AttnItem::half_block)
// at most 128 rows handled by two wave groups that take alternate tiles.  A launch of 256-row
// blocks uses it when some groups -- the last rows of a request -- fill at most half a block:
// such an item then holds its compute unit for half the time.
template <int SRC>
__global__ __launch_bounds__(512, 2) void attention_mfma_mixed_kernel(AttnArgs a)
{
    const bool half = a.inl.n ? false : a.items[blockIdx.x].half_block != 0;  // (regular launches have no half blocks)
    if (half) attention_body<4, SRC, 8, 2, false>(a);
    else attention_body<4, SRC, 8, 1, false>(a);
}

template <typename K> static int launch_kernel(K kernel, bool &attr_set, int lds_bytes, int threads, const AttnArgs &a, void *stream)
{
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kernel, dim3(a.n_items), dim3(threads), lds_bytes, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

template <int SRC, int NW, int KS, int STAGES, bool NTL> static int launch_variant_nt(const AttnArgs &a, void *stream)
{
    constexpr int lds_bytes = STAGES * STAGE_BYTES + (SRC == SRC_PAGED ? MAX_BLOCK_IDS * 4 : 0);
    static bool attr_set = false;
    return launch_kernel(attention_mfma_kernel<STAGES, SRC, NW, KS, NTL>, attr_set, lds_bytes, 64 * NW, a, stream);
}

// The streaming hint on the tile loads (a.nt_loads) exists for the 8-wave shapes, which stream
// long contexts; the planner asks for it nowhere else (launches of 4-wave workgroups are short or
// share their rows).
template <int SRC, int NW, int KS, int STAGES> static int launch_variant(const AttnArgs &a, void *stream)
{
    if (NW == 8 && a.nt_loads) return launch_variant_nt<SRC, NW, KS, STAGES, NW == 8>(a, stream);
    return launch_variant_nt<SRC, NW, KS, STAGES, false>(a, stream);
}

template <int SRC> static int launch_mixed(const AttnArgs &a, void *stream)
{
    constexpr int lds_bytes = 4 * STAGE_BYTES + (SRC == SRC_PAGED ? MAX_BLOCK_IDS * 4 : 0);
    static bool attr_set = false;
    return launch_kernel(attention_mfma_mixed_kernel<SRC>, attr_set, lds_bytes, 512, a, stream);
}

template <int NW, int KS, int STAGES> static int launch_nw(const AttnArgs &a, void *stream)
{
    if (a.tiles) return launch_variant<SRC_PACKETS, NW, KS, STAGES>(a, stream);
    return a.cache.layout != 0 ? launch_variant<SRC_PAGED, NW, KS, STAGES>(a, stream)
                               : launch_variant<SRC_CONTIG, NW, KS, STAGES>(a, stream);
}

// a.bm selects the row block: 256 packed rows (8 waves; a.mixed: with half blocks among them,
// see above) or 128.  128-row blocks run as 4 waves
// with two tile stages (two workgroups per CU), or -- a.split_in_wg, chosen when the launch
// has at most one item per CU -- as 8 waves in two groups that take alternate tiles.
int launch_attention_mfma(const AttnArgs &a, void *stream)
{
    if (a.d != D || (a.bm != 128 && a.bm != 256)) return (int)hipErrorInvalidValue;
    if (a.bm == 256 && a.mixed) {
        if (a.tiles) return launch_mixed<SRC_PACKETS>(a, stream);
        return a.cache.layout != 0 ? launch_mixed<SRC_PAGED>(a, stream) : launch_mixed<SRC_CONTIG>(a, stream);
    }
    if (a.bm == 256) return launch_nw<8, 1, 4>(a, stream);
    return a.split_in_wg ? launch_nw<8, 2, 4>(a, stream) : launch_nw<4, 1, 2>(a, stream);
}

}  // namespace kvp
