// kvp_plan.h -- plain-data plans the host builds per call and the kernels consume.
// Shared by the host runtime and the HIP kernels of this library only.
#pragma once
#include <stdint.h>

namespace kvp {

// The gather's plan is a list of segments: runs of rows of one retrieved packet that land in
// consecutive cache rows.  A workgroup takes one tile (up to AsmArgs::tile_rows rows) of one
// segment and finds it from blockIdx.x by the segments' cumulative tile counts.
//  - Whole packets: a segment is a packet, the same list serves every (layer, kv head), and
//    blockIdx.y selects those.
//  - Layered lists (requests with compressed packets, Sec. 5.4): the rows differ from layer to
//    layer, so a segment is one packet's rows in one layer and blockIdx.y selects the kv head.
struct AsmSeg {
    int64_t src_base;  // element offset in the arena: whole packets: the packet's K blob;
                       // layered: the first K row of kv head 0 in `layer`
    int32_t stride;    // rows between consecutive (layer, head) slices of the blob; negative (layered
                       // only): a compressed packet, -stride = the rows its layer kept, V follows that layer's K
    int32_t n_rows;    // rows of the segment (> 0)
    int32_t dst_row;   // cache row of the segment's first row
    int32_t pos;       // Delta_j: rotation offset of the packet (Eq. 1)
    int32_t req;       // request index
    int32_t layer;     // layered lists only
    int32_t tile0;     // index of the segment's first tile
    int32_t pad;
};
static_assert(sizeof(AsmSeg) == 40, "AsmSeg is 40 bytes");

constexpr int ASM_TILE_ROWS_MAX = 64;  // tiles hold 16, 32 or 64 rows

struct CacheView {
    void *k, *v;
    const int32_t *block_table;  // device, [n_req][max_blocks] (paged)
    int64_t req_stride;          // contig: elements between requests
    int64_t layer_stride;        // elements between layers (contig: per request; paged: pool)
    int32_t layout, t_cap, n_blocks, block_shift, max_blocks;
};

// Short lists ride in the kernel arguments (nothing is uploaded) and are scanned linearly.
// Longer ones are uploaded together with a map from tile to segment, so a workgroup finds its
// segment with two dependent loads whatever the length of the list.
constexpr int ASM_INLINE_SEGS = 80;

struct AsmArgs {
    const void *arena;
    const float2 *cs;    // [max_positions][d/2] (cos, sin)
    const AsmSeg *segs;  // device list, or nullptr: use `inline_seg`
    const int32_t *tile_seg;  // device, with `segs`: the segment of every tile
    CacheView cache;
    int32_t n_tiles, layer_begin, n_layers_total, n_kv, d;
    int32_t tile_rows, nontemporal;
    int32_t split_kv;  // grid.z = 2: a workgroup moves the K rows of its tile (z = 0) or the V rows (z = 1)
    int32_t layered;  // segments name their own layer; blockIdx.y = kv head
    int32_t n_segs;
    int32_t seg_tiles;  // > 0: every segment has this many tiles (segment of tile b = b / seg_tiles, no search)
    AsmSeg inline_seg[ASM_INLINE_SEGS];
};
static_assert(sizeof(AsmArgs) <= 4096, "kernel arguments are limited to 4 KB");

// ---- query prefill -------------------------------------------------------------
struct ReqMeta {
    int32_t ctx_len;  // rows already in this layer of the cache
    int32_t q_off;    // first query row in q / out
    int32_t n_q;
    int32_t pos0;     // position of query row 0 (= ctx_len unless compressed packets are in the context)
};

// Packed row m of a (request, kv head) pair: query token t = m / g, query head
// hq = h * g + m % g, so the g heads that share KV head h sit next to each other.
// A group is rows [m0, m0 + bm) of one pair; a work item is one kv range of a group.
struct AttnGroup {
    int32_t req, kv_head, m0, n_rows;  // n_rows <= bm
    int32_t part0, n_splits;           // partial slots part0 .. part0 + n_splits - 1 (part0 = group index x AttnArgs::part_stride)
    int32_t q_off, pad1;               // first row of the request in q / out
};
// Self-contained (one 64-byte read tells a workgroup everything it needs).
struct AttnItem {
    int32_t group, split, kv_begin, kv_end;  // kv rows [kv_begin, kv_end)
    int32_t req, kv_head, m0, n_rows;        // copy of the group
    int32_t ctx_len, q_off;                  // copy of the request
    int32_t part_slot;                       // partial slot to write, or -1: write `out` directly
    int32_t n_q;                             // query rows of the request
    int32_t pos0;                            // position of query row 0 (rows and positions differ with compressed packets)
    int32_t half_block;                      // MFMA kernel, launches of 256-row blocks: this group has at most 128 rows
    int32_t pad[2];
};
static_assert(sizeof(AttnItem) == 64, "AttnItem is 64 bytes");

// Attention straight from the packet store: one tile = up to 64 rows of one stored packet
// (kind 0) or of the request's own query rows (kind 1).
struct AttnTile {
    int64_t src_base;  // kind 0: element offset of the packet's K blob in the arena
    int32_t stride;    // kind 0: rows between (layer, head) slices of the blob; negative: a compressed packet,
                       // src_base is the called layer's own part and -stride the rows that layer kept
    int32_t row0;      // first row: inside the packet (kind 0) / among the query rows (kind 1)
    int32_t n_rows;    // 1..64
    int32_t pos;       // Delta_j of the packet; 0 for query rows
    int32_t kind;
    int32_t pad;
};
static_assert(sizeof(AttnTile) == 32, "AttnTile is 32 bytes");

// The work items of a launch for ONE request whose packed rows fit one row block are a regular
// pattern -- kv head h, split sp, all splits the same length but the last -- in a known launch
// order (the full splits of every head, head by head, then the heads' shorter last splits).  A
// workgroup of such a launch rebuilds its AttnItem from its index with scalar arithmetic and
// starts its query and tile loads one memory round trip earlier than one that first has to fetch
// its item.  The host fills this only after it has rebuilt every planned item with the same
// function and found it equal, field by field.  (A table of items in the kernel arguments was
// measured too: kernel arguments of 2 KB cost more per launch than the fetch they saved.)
struct AttnInline {
    int32_t n;                   // items of the launch (0: the items are read from memory)
    int32_t ctx_len, pos0, n_q;  // the request
    int32_t split_len;           // kv rows (in-place path: tiles) per split
    int32_t vis;                 // end of the kv range the rows may see
    int32_t ns, n_front;         // splits per head; how many of them come in the front part of the launch order
    int32_t n_rows;              // packed rows (n_q x heads per kv head)
};

__host__ __device__ inline AttnItem attn_inline_item(const AttnInline &t, int i, int n_kv, int part_stride)
{
    AttnItem it{};
    int h, sp;
    if (i < n_kv * t.n_front) {
        h = i / t.n_front;
        sp = i - h * t.n_front;
    } else {  // (n_front = ns - 1: the last splits follow, one per head)
        h = i - n_kv * t.n_front;
        sp = t.ns - 1;
    }
    it.group = h;
    it.split = sp;
    it.kv_begin = sp * t.split_len;
    it.kv_end = (sp + 1) * t.split_len < t.vis ? (sp + 1) * t.split_len : t.vis;
    it.req = 0;
    it.kv_head = h;
    it.m0 = 0;
    it.n_rows = t.n_rows;
    it.ctx_len = t.ctx_len;
    it.q_off = 0;
    it.part_slot = t.ns > 1 ? h * part_stride + sp : -1;
    it.n_q = t.n_q;
    it.pos0 = t.pos0;
    it.half_block = 0;
    return it;
}

struct AttnArgs {
    const void *q_rot;  // [tot_q][Hq][d], store dtype, rotated (generic kernel)
    // the MFMA kernel rotates the query and appends K_new / V_new itself:
    const void *q, *k_new, *v_new;  // un-rotated inputs of kvp_query_prefill
    const float2 *cs;               // [max_positions][d/2] (cos, sin)
    int32_t prerotated;
    // attention from the store without a cache (nullptr otherwise):
    const AttnTile *tiles;
    const void *arena;
    void *k_tail;  // [tot_q][n_kv][d]: rotated K_new, written by the kernel
    int32_t n_layers_total;
    CacheView cache;
    const ReqMeta *reqs;
    const AttnGroup *groups;
    const AttnItem *items;
    float *partials;  // [slot]: bm O~ rows of d elements, then m[bm], then l[bm] (fp32).  The rows are fp32, or
                      // (part_f16) fp16 scaled per row by a power of two that m and l carry along
    int32_t part_f16;
    void *out;        // [tot_q][Hq][d]
    int32_t n_items, n_groups, layer, n_q_heads, n_kv, d, bm, g;
    int32_t split_in_wg;  // MFMA kernel, 128-row blocks: two wave groups take alternate tiles
    int32_t mixed;        // MFMA kernel, 256-row blocks: some items are half blocks (AttnItem::half_block)
    int32_t nt_loads;     // MFMA kernel: no two work items read the same K/V rows, tiles are loaded with the streaming hint
    int32_t part_stride;  // partial slots per group
    int32_t max_group_rows;  // largest n_rows among the groups that are split (the combine grid covers no more)
    float scale_log2e;  // log2(e) / sqrt(d)
    AttnInline inl;     // MFMA kernel: the items as a formula (inl.n > 0), when the launch is that regular
};
static_assert(sizeof(AttnArgs) <= 4096, "kernel arguments are limited to 4 KB");

struct AppendArgs {
    const void *q, *k_new, *v_new;
    void *q_rot;
    const float2 *cs;
    CacheView cache;
    const ReqMeta *reqs;
    const int32_t *row_req;  // [tot_q] -> request
    int32_t tot_q, layer, n_q_heads, n_kv, d, prerotated;
    float q_scale;  // the rotated query is multiplied by this before it is stored
};

// Bytes of one partial slot and of its block of O~ rows.
__host__ __device__ inline int64_t part_rows_bytes(int bm, int d, int f16) { return (int64_t)bm * d * (f16 ? 2 : 4); }
__host__ __device__ inline int64_t part_slot_bytes(int bm, int d, int f16) { return part_rows_bytes(bm, d, f16) + (int64_t)bm * 8; }

// launchers (defined next to their kernels)
int launch_assemble(int dtype, const AsmArgs &a, int n_layers_launch, void *stream);
int launch_plan_upload(const void *host, void *dev, uint64_t bytes, void *stream);  // host: pinned, device-mapped
int launch_append(int dtype, const AppendArgs &a, void *stream);
int launch_attention(int dtype, const AttnArgs &a, int kernel_kind, void *stream);
int launch_combine(int dtype, const AttnArgs &a, void *stream);

enum { ATTN_GENERIC = 0, ATTN_MFMA = 1 };

// MFMA kernel, paged layout: an item's block ids live in LDS, so one item may span at most
// this many blocks, and blocks must hold at least MFMA_MIN_BLOCK_SIZE rows.
constexpr int MFMA_MAX_ITEM_BLOCKS = 2048;
constexpr int MFMA_MIN_BLOCK_SIZE = 16;

}  // namespace kvp
