// kvp_runtime.hip -- host runtime behind the C ABI: packet directory over the caller's
// arena, the host-built cos/sin table, per-call plans (offsets Delta_j, gather tiles,
// attention groups / split-KV items, block tables) and the kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <unordered_set>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "../../include/kvp.h"
#include "kvp_plan.h"

using namespace kvp;

namespace {

constexpr uint64_t ALIGN = 256;
inline uint64_t align_up(uint64_t x, uint64_t a = ALIGN) { return (x + a - 1) / a * a; }

struct PacketRec {
    int64_t elem_off;  // element offset of the blob in the arena
    int32_t n_tokens;  // rows (positions) of the packet
    int32_t stride;    // rows between (layer, head) slices: n_tokens + slice padding
    // compressed packets only: rows kept per layer and the element offset of each layer's
    // part of the blob ([K: Hkv x rows][V: Hkv x rows], layer after layer)
    std::vector<int32_t> rows;
    std::vector<int64_t> layer_off;
    // packets stored without their header rows: the first head_rows positions come from the
    // store's shared header blob, the blob at elem_off holds the n_tokens - head_rows others
    int32_t head_rows = 0;
    bool compressed() const { return !rows.empty(); }
    int body_rows() const { return n_tokens - head_rows; }
};

// A pinned-host / device twin buffer that carries one call's plan.  It is rewritten only
// after the work that read it has finished (event recorded behind that work).
struct PlanSlot {
    char *host = nullptr;
    char *dev = nullptr;
    uint64_t cap = 0;
    hipEvent_t ev = nullptr;
    bool pending = false;

    int ensure(uint64_t bytes, bool dry)
    {
        if (dry) {
            if (cap < bytes) {
                free(host);
                host = (char *)malloc(bytes);
                cap = bytes;
            }
            return 0;
        }
        if (pending) {
            hipError_t e = hipEventSynchronize(ev);
            if (e != hipSuccess) return (int)e;
            pending = false;
        }
        if (!ev) {
            hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
            if (e != hipSuccess) return (int)e;
        }
        if (cap < bytes) {
            uint64_t want = std::max<uint64_t>(align_up(bytes, 4096), 1 << 16);
            if (host) (void)hipHostFree(host);
            if (dev) (void)hipFree(dev);
            host = dev = nullptr;
            cap = 0;
            hipError_t e = hipHostMalloc((void **)&host, want, hipHostMallocDefault);
            if (e != hipSuccess) return (int)e;
            e = hipMalloc((void **)&dev, want);
            if (e != hipSuccess) return (int)e;
            cap = want;
        }
        return 0;
    }
    void release(bool dry)
    {
        if (dry) {
            free(host);
        } else {
            if (pending) (void)hipEventSynchronize(ev);
            if (host) (void)hipHostFree(host);
            if (dev) (void)hipFree(dev);
            if (ev) (void)hipEventDestroy(ev);
        }
        *this = PlanSlot();
    }
};

// Ring of plan buffers for kvp_assemble.  A slot remembers the plan it holds (its bytes and the
// stream it was uploaded on): a call that would upload the same bytes again -- the same requests
// on the same cache geometry, as in a serving loop that re-assembles after an eviction, or a
// benchmark's repeated step -- launches from the copy already on the device instead.
struct PlanRing {
    static constexpr int SLOTS = 8;
    struct Slot : PlanSlot {
        std::vector<char> image;  // the bytes in `dev` (empty: none)
        void *stream = nullptr;
        bool used_since_event = false;  // launches newer than `ev` may still read `dev`
    };
    Slot slot[SLOTS];
    int next = 0;
    bool dry = false;

    Slot *find(const std::vector<char> &image, void *stream)
    {
        for (auto &s : slot)
            if (!s.image.empty() && s.stream == stream && s.image.size() == image.size() &&
                memcmp(s.image.data(), image.data(), image.size()) == 0)
                return &s;
        return nullptr;
    }
    // The next slot, ready to be rewritten: work that may still read it is waited for.
    int acquire(uint64_t bytes, Slot **out)
    {
        Slot &s = slot[next];
        next = (next + 1) % SLOTS;
        *out = &s;
        s.image.clear();
        if (!dry && s.used_since_event) {
            s.used_since_event = false;
            hipError_t rc = s.ev ? hipEventRecord(s.ev, (hipStream_t)s.stream) : hipErrorInvalidHandle;
            if (rc == hipSuccess) {
                s.pending = true;
            } else {
                (void)hipGetLastError();
                rc = hipDeviceSynchronize();
                if (rc != hipSuccess) return (int)rc;
                s.pending = false;
            }
        }
        return s.ensure(bytes, dry);
    }
    bool unsettled() const
    {
        for (auto &s : slot)
            if (s.used_since_event) return true;
        return false;
    }
    void release()
    {
        for (auto &s : slot) {
            s.release(dry);
            s.image.clear();
            s.used_since_event = false;
        }
    }
};

thread_local std::string g_create_error;

}  // namespace

// ---- scratch of the entry point that allocates nothing (kvp_query_prefill_static) ----------
// One array per GPU, held by every GPU the library runs on until the process ends: the plan of
// the last call in its first KVP_STATIC_PLAN_BYTES, then the workspace (rotated query, split-KV
// partials).  In host code the array's name is only a stand-in: the device address comes from
// hipGetSymbolAddress, once per device, and is what every launch and copy gets.
#define KVP_STATIC_SCRATCH_BYTES (32ull << 20)
#define KVP_STATIC_PLAN_BYTES (1ull << 20)
static __device__ __align__(256) unsigned char scratch[KVP_STATIC_SCRATCH_BYTES];

struct kvp_store {
    kvp_config_t cfg;
    std::vector<float> inv_freq;
    std::unordered_map<int64_t, PacketRec> dir;
    uint64_t used_bytes = 0;
    float2 *cs_dev = nullptr;
    void *arena_dev = nullptr;  // the arena as the kernels address it
    bool arena_host = false;    // the arena is pinned host memory mapped into the device (read over PCIe)
    PacketRec header;       // the header rows stored once (kvp_store_put_header); n_tokens 0: none
    PlanRing ring;          // plans of kvp_assemble
    // The prefill plan depends only on the request geometry (context lengths, query
    // offsets, block table), which is the same for every layer of a forward pass: the
    // uploaded plan is kept and reused while that geometry does not change.  With compressed
    // packets every layer has its own row counts, hence its own plan: kvp_query_prefill keeps
    // a set of plans (one more than the layers, at least PlanRing::SLOTS), each in a buffer
    // of its own, replaced least recently used first; kvp_prefill_packets likewise.
    struct PrefillCached {
        bool valid = false;
        std::vector<int32_t> sig;
        uint64_t sig_hash = 0, last_use = 0;
        PlanSlot own;               // kvp_query_prefill: the entry's own buffer
        PlanSlot *slot = nullptr;   // the buffer the plan is in
        void *stream = nullptr;
        const ReqMeta *reqs_dev = nullptr;
        const int32_t *row_req_dev = nullptr, *bt_dev = nullptr;
        const AttnGroup *groups_dev = nullptr;
        const AttnItem *items_dev = nullptr;
        const AttnTile *tiles_dev = nullptr;
        int kind = 0, bm = 0, n_items = 0, n_groups = 0, bt_stride = 0, tot_q = 0, part_stride = 1, max_group_rows = 0;
        bool any_split = false, mixed = false, split_in_wg = false, shared_rows = false;
        AttnInline inl{};       // the items as kernel arguments (inl.n = 0: not applicable)
        bool captured = false;  // a HIP graph launches from this plan: the entry is never replaced
        uint64_t owner = 0;     // the static scratch's entry only: serial of the store whose plan it holds
        // Launches from a kept plan record no event (an event per layer costs a marker packet
        // between the kernels and a microsecond of host time); the entry remembers that work
        // newer than its event may still read the plan, and settles that when it is replaced.
        bool used_since_event = false;
        uint64_t need = 0;
    };
    uint64_t serial = 0;  // distinguishes this store from any other the process has had
    std::deque<PrefillCached> pf_set;  // kvp_query_prefill
    std::deque<PrefillCached> pk_set;  // kvp_prefill_packets
    uint64_t pf_clock = 0;
    std::vector<int32_t> sig_scratch;
    std::vector<char> asm_image;  // the gather plan of the current call, as it would be uploaded
    std::string err;
    std::vector<AsmSeg> dbg_segs;  // the last gather plan (kvp_debug_last_plan)
    bool dbg_layered = false;
    // the last prefill plan, kept as built (kvp_debug_last_plan expands it on request)
    struct DebugPlan {
        int64_t head[6] = {0, 0, 0, 0, 0, 0};  // kind, bm, groups, items, slots, workspace bytes needed
        std::vector<AttnGroup> groups;
        std::vector<AttnItem> items;
        std::vector<AttnTile> tiles;
        bool has_tiles = false;
        int64_t inl_n = 0;  // items that ride in the kernel arguments (0: none)
    } dbg_plan;
    bool dry = false;
    int n_cu = 256;
    int force_generic = 0;
    int target_items = 0;  // 0: three quarters of the CU count (measured optimum at 8K context)
    int asm_tile_rows = 0;  // 0: chosen per call (tile_rows_for)
    int asm_nontemporal = -1;  // -1: non-temporal gather decided per call
    int asm_split_kv = 1;  // the gather's workgroups move either the K or the V rows of a tile (KVP_ASM_SPLIT_KV=0: both)
    int dbg_tile_rows = 32;  // tile rows of the last gather plan
    int nt_loads = -1;  // test knob (KVP_ATTN_NT_LOADS=0/1): streaming hint on the attention kernel's tile loads
    int mixed_blocks = 1;  // test knob (KVP_ATTN_MIXED=0): no half blocks in launches of 256-row blocks
    int plan_copy_engine = 0;  // test knob: plans go up with hipMemcpyAsync instead of the upload kernel
    int inline_items = 1;  // test knob (KVP_ATTN_INLINE_ITEMS=0): work items are always read from memory
    int force_bm = 0;  // test knob: row-block size of the MFMA attention kernel
    int force_split_in_wg = -1;  // test knob: 0 / 1 forces the 4-wave / 8-wave-in-two-groups shape of 128-row blocks
    size_t esize = 2;
};

namespace {

// Per-device state of the static scratch: its device address, a pinned staging buffer for the
// plan and an event behind the last upload, all made at set-up (kvp_store_create), never freed.
constexpr int MAX_DEVICES = 64;
struct StaticScratch {
    char *ptr = nullptr;               // device address of `scratch` on this GPU
    kvp_store::PrefillCached entry;    // the plan the scratch holds (entry.own: staging buffer / scratch / event)
    bool ready = false;
};
StaticScratch g_static[MAX_DEVICES];
uint64_t g_store_serial = 0;

// Once per device, with that device current.
hipError_t static_scratch_setup(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    StaticScratch &ss = g_static[device];
    if (ss.ready) return hipSuccess;
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || ((uintptr_t)p & (ALIGN - 1))) return hipErrorInvalidSymbol;
    PlanSlot &slot = ss.entry.own;
    e = hipHostMalloc((void **)&slot.host, KVP_STATIC_PLAN_BYTES, hipHostMallocDefault);
    if (e != hipSuccess) return e;
    e = hipEventCreateWithFlags(&slot.ev, hipEventDisableTiming);
    if (e != hipSuccess) {
        (void)hipHostFree(slot.host);
        slot.host = nullptr;
        return e;
    }
    slot.dev = (char *)p;
    slot.cap = KVP_STATIC_PLAN_BYTES;
    ss.ptr = (char *)p;
    ss.ready = true;
    return hipSuccess;
}

int fail(kvp_store *s, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (s) s->err = buf;
    else g_create_error = buf;
    return code;
}

int hip_fail(kvp_store *s, hipError_t e, const char *what)
{
    return fail(s, KVP_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(s, call)                                          \
    do {                                                          \
        hipError_t e_ = (call);                                   \
        if (e_ != hipSuccess) return hip_fail((s), e_, #call);    \
    } while (0)

// Is the stream being captured into a HIP graph?  (The null stream cannot be.)  Launches made
// then run later, any number of times: nothing they read may be rewritten, and no event of
// the library may be recorded into the graph.
bool capturing(const kvp_store *s, void *hip_stream)
{
    if (s->dry || !hip_stream) return false;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)hip_stream, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs == hipStreamCaptureStatusActive;
}

bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }
int ilog2(int x) { int s = 0; while ((1 << s) < x) ++s; return s; }

// (cos, sin) of pos * theta_i for every position: double libm, rounded to fp32.
void build_cos_sin(const std::vector<float> &inv_freq, int max_pos, std::vector<float2> &out)
{
    const int half = (int)inv_freq.size();
    out.resize((size_t)max_pos * half);
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<unsigned>(hw ? hw : 1, 16);
    if ((int64_t)max_pos * half < (1 << 16)) nt = 1;
    auto work = [&](int t) {
        for (int p = t; p < max_pos; p += nt)
            for (int i = 0; i < half; ++i) {
                double a = (double)p * (double)inv_freq[i];
                out[(size_t)p * half + i] = make_float2((float)cos(a), (float)sin(a));
            }
    };
    if (nt == 1) { work(0); return; }
    std::vector<std::thread> th;
    for (int t = 0; t < nt; ++t) th.emplace_back(work, t);
    for (auto &t : th) t.join();
}

struct CacheCheck {
    int shift = 0;
    int64_t cap_rows = 0;  // rows a request can hold
};

int check_cache(kvp_store *s, const kvp_cache_t *c, int n_req, CacheCheck &cc)
{
    if (!c) return fail(s, KVP_E_INVAL, "cache is null");
    if (c->layout != KVP_CONTIG && c->layout != KVP_PAGED) return fail(s, KVP_E_INVAL, "unknown cache layout %d", c->layout);
    if (!c->k || !c->v) return fail(s, KVP_E_INVAL, "cache k/v pointer is null");
    if (((uintptr_t)c->k | (uintptr_t)c->v) & 15) return fail(s, KVP_E_INVAL, "cache k/v must be 16-byte aligned");
    if (!c->ctx_len && n_req > 0) return fail(s, KVP_E_INVAL, "cache ctx_len is null");
    if (c->layout == KVP_CONTIG) {
        if (c->t_cap < 0) return fail(s, KVP_E_INVAL, "t_cap < 0");
        cc.cap_rows = c->t_cap;
    } else {
        if (!is_pow2(c->block_size)) return fail(s, KVP_E_INVAL, "block_size must be a power of two");
        if (c->n_blocks < 0 || c->max_blocks_per_req < 0) return fail(s, KVP_E_INVAL, "negative block counts");
        if (!c->block_table && n_req > 0 && c->max_blocks_per_req > 0) return fail(s, KVP_E_INVAL, "block_table is null");
        cc.shift = ilog2(c->block_size);
        cc.cap_rows = (int64_t)c->max_blocks_per_req * c->block_size;
    }
    return 0;
}

// Copies the first n_blk[r] table entries of every request into a compact
// [n_req][stride] table, checking the block ids.
int compact_block_table(kvp_store *s, const kvp_cache_t *c, int n_req, const std::vector<int> &first_blk,
                        const std::vector<int> &n_blk, int stride, int32_t *dst)
{
    for (int r = 0; r < n_req; ++r) {
        const int32_t *row = c->block_table + (int64_t)r * c->max_blocks_per_req;
        for (int b = 0; b < stride; ++b) dst[(int64_t)r * stride + b] = 0;
        for (int b = first_blk[r]; b < n_blk[r]; ++b) {
            if (row[b] < 0 || row[b] >= c->n_blocks)
                return fail(s, KVP_E_INVAL, "block_table[%d][%d] = %d is outside [0, %d)", r, b, row[b], c->n_blocks);
            dst[(int64_t)r * stride + b] = row[b];
        }
    }
    return 0;
}

CacheView make_view(const kvp_store *s, const kvp_cache_t *c, int shift, const int32_t *bt_dev, int bt_stride)
{
    const kvp_config_t &g = s->cfg;
    CacheView v;
    v.k = c->k;
    v.v = c->v;
    v.block_table = bt_dev;
    v.layout = c->layout;
    v.t_cap = c->t_cap;
    v.n_blocks = c->n_blocks;
    v.block_shift = shift;
    v.max_blocks = bt_stride;
    if (c->layout == KVP_CONTIG) {
        v.layer_stride = (int64_t)g.n_kv_heads * c->t_cap * g.head_dim;
        v.req_stride = v.layer_stride * g.n_layers;
    } else {
        v.layer_stride = (int64_t)c->n_blocks * g.n_kv_heads * c->block_size * g.head_dim;
        v.req_stride = 0;
    }
    return v;
}

// Sub-allocator over one plan slot.
struct PlanWriter {
    char *host, *dev;
    uint64_t off = 0;
    template <typename T> T *put(uint64_t n, const T **dev_ptr)
    {
        off = align_up(off, 64);
        T *h = (T *)(host + off);
        *dev_ptr = (const T *)(dev ? dev + off : host + off);
        off += n * sizeof(T);
        return h;
    }
};

// Sends a plan from its slot's host buffer to the device twin, in stream order.
int upload_plan(kvp_store *s, PlanSlot *slot, uint64_t bytes, void *hip_stream)
{
    if (s->plan_copy_engine) {
        HIP_TRY(s, hipMemcpyAsync(slot->dev, slot->host, bytes, hipMemcpyHostToDevice, (hipStream_t)hip_stream));
        return KVP_OK;
    }
    int e = launch_plan_upload(slot->host, slot->dev, bytes, hip_stream);
    if (e) return hip_fail(s, (hipError_t)e, "plan upload");
    return KVP_OK;
}

// Does a gather of `rows` context rows per layer, of which `unique_rows` come from distinct
// packets, stream far more than the last-level cache holds, nearly all of it read once?  Then
// its loads and stores carry the non-temporal hint.  Measured (us per layer, assemble + prefill):
// one request of 2.9K rows x 32 layers 26.97 -> 25.74, 8K rows 37.85 -> 37.48, 8 requests of 16.9K
// rows x 4 layers 500.8 -> 482.7 -- the gather itself is no faster, the attention that follows
// is, finding fewer dirty lines in its way; a batch whose popular packets are gathered several
// times loses the reuse (1107 -> 1187), and a 67 MB call that the attention reads right back
// out of the cache is slower too (49 -> 54).
bool gather_streams_once(const kvp_store *s, int64_t rows, int64_t unique_rows, int n_layers)
{
    const int64_t bytes = 4 * rows * n_layers * s->cfg.n_kv_heads * s->cfg.head_dim * (int64_t)s->esize;  // K and V, read and written
    return bytes >= (512ll << 20) && unique_rows * 10 >= rows * 9;
}

// Tiles of `rows` rows at the store's tile size.
int tiles_of(int rows, int tile_rows) { return (rows + tile_rows - 1) / tile_rows; }

// Rows per gather tile.  Measured with workgroups that move either K or V: 32 rows (8 KB in,
// 8 KB out per workgroup) on a contiguous cache -- one 8K request x 32 layers 382 -> 365 us, eight
// 16.9K requests x 4 layers 795 -> 783 us, against 374 and 788 with 64 rows -- and 64 rows on a
// paged cache, where every row's block is looked up (64 requests, 290K rows: 352 -> 342 us, with
// 32 rows 385).
int tile_rows_for(const kvp_store *s, const kvp_cache_t *cache)
{
    if (s->asm_tile_rows) return s->asm_tile_rows;
    return cache->layout == KVP_PAGED ? 64 : 32;
}

// Uploads a gather plan (segment list, block table) if it does not fit the kernel arguments,
// and launches the gather: grid = (tiles, layers x kv heads), or (tiles, kv heads) for a
// layered list.
int run_gather(kvp_store *s, const std::vector<AsmSeg> &segs, int64_t n_tiles, int tile_rows, bool layered, int layer_begin,
               int n_layers_launch, const kvp_cache_t *cache, const CacheCheck &cc, int n_req,
               const std::vector<int> &first_blk, const std::vector<int> &n_blk, bool streams_once, void *hip_stream)
{
    const kvp_config_t &g = s->cfg;
    if (n_tiles > 0x7fffffff) return fail(s, KVP_E_CAPACITY, "%lld gather tiles in one call", (long long)n_tiles);
    int bt_stride = 0;
    for (int r = 0; r < n_req; ++r) bt_stride = std::max(bt_stride, n_blk[r]);
    const bool inline_plan = (int)segs.size() <= ASM_INLINE_SEGS && cache->layout == KVP_CONTIG;
    const AsmSeg *segs_dev = nullptr;
    const int32_t *bt_dev = nullptr, *tile_seg_dev = nullptr;
    PlanRing::Slot *slot = nullptr;
    uint64_t upload = 0;
    if (!s->dry) HIP_TRY(s, hipSetDevice(g.device));
    if (!inline_plan && capturing(s, hip_stream))
        return fail(s, KVP_E_INVAL, "kvp_assemble under stream capture: only calls whose plan rides in the kernel arguments "
                                    "(contiguous cache, at most %d segments) can be captured", ASM_INLINE_SEGS);
    bool kept = false;  // the plan is on the device already (a slot holds the same bytes)
    if (!inline_plan) {
        const uint64_t bytes = align_up(segs.size() * sizeof(AsmSeg), 64) + align_up((uint64_t)n_tiles * 4, 64) +
                               (uint64_t)n_req * bt_stride * 4 + 256;
        std::vector<char> &image = s->asm_image;
        image.assign(bytes, 0);
        PlanWriter w{image.data(), nullptr};
        const AsmSeg *segs_at = nullptr;
        const int32_t *ts_at = nullptr, *bt_at = nullptr;
        AsmSeg *sh = w.put<AsmSeg>(segs.size(), &segs_at);
        if (!segs.empty()) memcpy(sh, segs.data(), segs.size() * sizeof(AsmSeg));
        int32_t *ts = w.put<int32_t>((uint64_t)n_tiles, &ts_at);
        for (size_t i = 0; i < segs.size(); ++i) {
            const int32_t end = i + 1 < segs.size() ? segs[i + 1].tile0 : (int32_t)n_tiles;
            for (int32_t t = segs[i].tile0; t < end; ++t) ts[t] = (int32_t)i;
        }
        if (cache->layout == KVP_PAGED && bt_stride > 0) {
            int32_t *bh = w.put<int32_t>((uint64_t)n_req * bt_stride, &bt_at);
            int rc = compact_block_table(s, cache, n_req, first_blk, n_blk, bt_stride, bh);
            if (rc) return rc;
        }
        upload = w.off;
        image.resize(upload);
        slot = s->dry ? nullptr : s->ring.find(image, hip_stream);
        kept = slot != nullptr;
        if (!kept) {
            int hrc = s->ring.acquire(upload, &slot);
            if (hrc) return hip_fail(s, (hipError_t)hrc, "plan buffer");
            memcpy(slot->host, image.data(), upload);
        }
        // where the pieces are on the device (dry stores: in the slot's host buffer)
        const char *at = s->dry ? slot->host : slot->dev;
        segs_dev = (const AsmSeg *)(at + ((const char *)segs_at - image.data()));
        tile_seg_dev = (const int32_t *)(at + ((const char *)ts_at - image.data()));
        bt_dev = bt_at ? (const int32_t *)(at + ((const char *)bt_at - image.data())) : nullptr;
    }
    s->dbg_segs = segs;
    s->dbg_layered = layered;
    s->dbg_tile_rows = tile_rows;
    if (s->dry || n_tiles == 0 || n_layers_launch <= 0) return KVP_OK;

    hipStream_t st = (hipStream_t)hip_stream;
    AsmArgs a;
    a.arena = s->arena_dev;
    a.cs = s->cs_dev;
    a.segs = nullptr;
    a.n_segs = (int)segs.size();
    a.tile_seg = nullptr;
    a.layered = layered ? 1 : 0;
    a.seg_tiles = 0;
    if (inline_plan) {
        for (size_t i = 0; i < segs.size(); ++i) a.inline_seg[i] = segs[i];
        // equal tile counts (packets of one length): a workgroup finds its segment by division
        const int64_t per = segs.empty() ? 0 : n_tiles / (int64_t)segs.size();
        bool uniform = per > 0 && per * (int64_t)segs.size() == n_tiles;
        for (size_t i = 0; uniform && i < segs.size(); ++i) uniform = segs[i].tile0 == (int64_t)i * per;
        if (uniform) a.seg_tiles = (int32_t)per;
    } else {
        if (!kept) {
            int urc = upload_plan(s, slot, upload, hip_stream);
            if (urc) return urc;
        }
        a.segs = segs_dev;
        a.tile_seg = tile_seg_dev;
    }
    a.cache = make_view(s, cache, cc.shift, bt_dev, bt_stride);
    a.n_tiles = (int)n_tiles;
    a.tile_rows = tile_rows;
    a.nontemporal = s->asm_nontemporal >= 0 ? s->asm_nontemporal : (streams_once ? 1 : 0);
    a.split_kv = s->asm_split_kv;
    a.layer_begin = layer_begin;
    a.n_layers_total = g.n_layers;
    a.n_kv = g.n_kv_heads;
    a.d = g.head_dim;
    int e = launch_assemble(g.dtype, a, layered ? 1 : n_layers_launch, hip_stream);
    if (e) return hip_fail(s, (hipError_t)e, "assemble launch");
    if (slot && kept) {
        slot->used_since_event = true;  // (no event per launch: settled when the slot is rewritten)
    } else if (slot) {
        HIP_TRY(s, hipEventRecord(slot->ev, st));
        slot->pending = true;
        slot->image = s->asm_image;  // from now on the slot can serve the same plan again
        slot->stream = hip_stream;
    }
    return KVP_OK;
}

// kvp_assemble for requests with compressed packets (Sec. 5.4): positions advance by the
// packets' spans, rows by what each layer kept, so every (packet, layer) is a segment of its
// own, and one launch covers (tile, kv head).
int assemble_compressed(kvp_store *s, const kvp_request_t *reqs, int n_req, int layer_begin, int layer_end,
                        kvp_cache_t *cache, const CacheCheck &cc, void *hip_stream)
{
    const kvp_config_t &g = s->cfg;
    if (!cache->ctx_rows) return fail(s, KVP_E_INVAL, "compressed packets need kvp_cache_t.ctx_rows");
    const int n_l = layer_end - layer_begin;
    const int tile_rows = tile_rows_for(s, cache);
    std::vector<AsmSeg> segs;
    int64_t n_tiles = 0, rows_total = 0, rows_unique = 0;  // (rows of the first layer asked for stand for all)
    std::unordered_set<int64_t> seen;
    std::vector<int> pos_end(n_req), first_blk(n_req, 0), n_blk(n_req, 0);
    std::vector<int64_t> rows_end((size_t)n_req * std::max(n_l, 1), 0);
    for (int r = 0; r < n_req; ++r) {
        const kvp_request_t &q = reqs[r];
        if (q.base_pos < 0) return fail(s, KVP_E_INVAL, "request %d: base_pos %d < 0", r, q.base_pos);
        int64_t pos = q.base_pos, max_rows = q.base_pos;
        std::vector<int64_t> row(std::max(n_l, 1), q.base_pos);  // the caller's rows below base_pos are not compressed
        for (int j = 0; j < q.k; ++j) {
            auto it = s->dir.find(q.packet_ids[j]);
            if (it == s->dir.end()) return fail(s, KVP_E_NOTFOUND, "request %d: packet %lld not in the store", r, (long long)q.packet_ids[j]);
            const PacketRec &p = it->second;
            if (pos + p.n_tokens > g.max_positions)
                return fail(s, KVP_E_CAPACITY, "request %d: context exceeds max_positions %d", r, g.max_positions);
            if (n_l > 0) {
                const int n0 = p.compressed() ? p.rows[layer_begin] : p.n_tokens;
                rows_total += n0;
                if (seen.insert(q.packet_ids[j]).second) rows_unique += n0;
            }
            for (int li = 0; li < n_l; ++li) {
                const int l = layer_begin + li;
                // src: first K row of head 0 in this layer; a negative stride marks a blob laid out layer by layer
                auto emit = [&](int64_t src, int stride, int n) {
                    if (n == 0) return;
                    segs.push_back(AsmSeg{src, stride, n, (int32_t)row[li], (int32_t)pos, r, l, (int32_t)n_tiles, 0});
                    n_tiles += tiles_of(n, tile_rows);
                    row[li] += n;
                };
                const int64_t slices = (int64_t)l * g.n_kv_heads * g.head_dim;  // x stride = elements before layer l
                if (p.compressed()) {
                    emit(p.layer_off[l], -p.rows[l], p.rows[l]);
                } else {
                    if (p.head_rows) emit(s->header.elem_off + slices * s->header.stride, s->header.stride, p.head_rows);
                    emit(p.elem_off + slices * p.stride, p.stride, p.body_rows());
                }
            }
            pos += p.n_tokens;
        }
        for (int li = 0; li < n_l; ++li) {
            rows_end[(size_t)r * n_l + li] = row[li];
            max_rows = std::max(max_rows, row[li]);
        }
        if (max_rows > cc.cap_rows) return fail(s, KVP_E_CAPACITY, "request %d: %lld rows do not fit the cache (%lld)", r, (long long)max_rows, (long long)cc.cap_rows);
        pos_end[r] = (int)pos;
        if (cache->layout == KVP_PAGED && max_rows > q.base_pos) {
            first_blk[r] = q.base_pos >> cc.shift;
            n_blk[r] = (int)((max_rows - 1) >> cc.shift) + 1;
        }
    }
    int rc = run_gather(s, segs, n_tiles, tile_rows, true, layer_begin, n_l, cache, cc, n_req, first_blk, n_blk,
                        gather_streams_once(s, rows_total, rows_unique, n_l), hip_stream);
    if (rc) return rc;
    for (int r = 0; r < n_req; ++r) {
        cache->ctx_len[r] = pos_end[r];
        for (int li = 0; li < n_l; ++li)
            cache->ctx_rows[(int64_t)r * g.n_layers + layer_begin + li] = (int32_t)rows_end[(size_t)r * n_l + li];
    }
    return KVP_OK;
}

}  // namespace

// =====================================================================================
extern "C" {

const char *kvp_version(void) { return "kvp 0.1 gfx950"; }

const char *kvp_last_error(const kvp_store_t *store) { return store ? store->err.c_str() : g_create_error.c_str(); }

uint64_t kvp_packet_bytes(const kvp_config_t *cfg, int32_t n_tokens)
{
    if (!cfg || n_tokens < 0) return 0;
    uint64_t es = cfg->dtype == KVP_BF16 ? 2 : 4;
    return align_up(2ull * cfg->n_layers * cfg->n_kv_heads * (uint64_t)n_tokens * cfg->head_dim * es);
}

int kvp_store_create(const kvp_config_t *cfg, kvp_store_t **out)
{
    if (!cfg || !out) return fail(nullptr, KVP_E_INVAL, "cfg or out is null");
    if (cfg->n_layers < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1)
        return fail(nullptr, KVP_E_INVAL, "n_layers, n_q_heads, n_kv_heads must be >= 1");
    if (cfg->n_q_heads % cfg->n_kv_heads) return fail(nullptr, KVP_E_INVAL, "n_q_heads must be a multiple of n_kv_heads");
    if (cfg->head_dim < 2 || cfg->head_dim > 256 || (cfg->head_dim & 1))
        return fail(nullptr, KVP_E_INVAL, "head_dim must be even and in [2, 256]");
    if (cfg->dtype != KVP_F32 && cfg->dtype != KVP_BF16) return fail(nullptr, KVP_E_INVAL, "unknown dtype %d", cfg->dtype);
    if (cfg->n_header < 0 || cfg->n_trailer < 0) return fail(nullptr, KVP_E_INVAL, "negative adapter length");
    if (cfg->max_positions < 1 || cfg->max_positions > (1 << 21)) return fail(nullptr, KVP_E_INVAL, "max_positions must be in [1, 2^21]");
    if (!cfg->inv_freq && !(cfg->rope_base > 0.0)) return fail(nullptr, KVP_E_INVAL, "rope_base must be positive");
    const bool dry = cfg->device == KVP_DEVICE_NONE;
    if (!dry) {
        if (cfg->device < 0) return fail(nullptr, KVP_E_INVAL, "bad device %d", cfg->device);
        if (!cfg->arena && cfg->arena_bytes) return fail(nullptr, KVP_E_INVAL, "arena is null");
        if ((uintptr_t)cfg->arena & (ALIGN - 1)) return fail(nullptr, KVP_E_INVAL, "arena must be 256-byte aligned");
    }
    kvp_store *s = new kvp_store();
    s->cfg = *cfg;
    s->serial = ++g_store_serial;
    s->dry = dry;
    s->ring.dry = dry;
    s->esize = cfg->dtype == KVP_BF16 ? 2 : 4;
    const int half = cfg->head_dim / 2;
    s->inv_freq.resize(half);
    for (int i = 0; i < half; ++i)
        s->inv_freq[i] = cfg->inv_freq ? cfg->inv_freq[i]
                                       : (float)pow(cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
    s->cfg.inv_freq = nullptr;
    const char *fg = getenv("KVP_FORCE_GENERIC_ATTENTION");
    s->force_generic = fg && fg[0] == '1';
    const char *tr = getenv("KVP_ASM_TILE_ROWS");  // tuning knobs of the gather kernel
    if (tr && (atoi(tr) == 16 || atoi(tr) == 32 || atoi(tr) == 64)) s->asm_tile_rows = atoi(tr);
    if (const char *sk = getenv("KVP_ASM_SPLIT_KV")) s->asm_split_kv = sk[0] != '0';
    if (cfg->head_dim != 64 && cfg->head_dim != 128 && cfg->head_dim != 256) s->asm_split_kv = 0;  // (the scalar kernel moves both)
    const char *nt = getenv("KVP_ASM_NONTEMPORAL");
    if (nt) s->asm_nontemporal = nt[0] == '1';  // unset: decided per call (run_gather)
    if (const char *pc = getenv("KVP_PLAN_COPY_ENGINE")) s->plan_copy_engine = pc[0] == '1';
    if (const char *mb = getenv("KVP_ATTN_MIXED")) s->mixed_blocks = mb[0] != '0';
    if (const char *nl = getenv("KVP_ATTN_NT_LOADS")) s->nt_loads = nl[0] != '0';
    if (const char *fb = getenv("KVP_ATTN_BM")) s->force_bm = atoi(fb);
    if (const char *ii = getenv("KVP_ATTN_INLINE_ITEMS")) s->inline_items = ii[0] != '0';
    if (const char *fd = getenv("KVP_ATTN_SPLIT_IN_WG")) s->force_split_in_wg = atoi(fd) != 0;
    const char *ti = getenv("KVP_ATTN_TARGET_ITEMS");  // test knob: how finely split-KV cuts
    if (ti && atoi(ti) > 0) s->target_items = std::min(atoi(ti), 1 << 16);
    if (!dry) {
        hipError_t e = hipSetDevice(cfg->device);
        if (e == hipSuccess) {
            hipDeviceProp_t prop;
            if (hipGetDeviceProperties(&prop, cfg->device) == hipSuccess && prop.multiProcessorCount > 0)
                s->n_cu = prop.multiProcessorCount;
            // The arena is device memory, or pinned host memory that the device can address
            // (the paper's own tier, Sec. 5.1: packets wait in CPU memory).
            s->arena_dev = cfg->arena;
            if (cfg->arena) {
                hipPointerAttribute_t attr;
                hipError_t pe = hipPointerGetAttributes(&attr, cfg->arena);
                if (pe == hipSuccess && attr.type == hipMemoryTypeHost && attr.devicePointer) {
                    s->arena_host = true;
                    s->arena_dev = attr.devicePointer;
                } else if (pe != hipSuccess || attr.type != hipMemoryTypeDevice) {
                    (void)hipGetLastError();
                    delete s;
                    return fail(nullptr, KVP_E_INVAL, "arena must be device memory or pinned (device-mapped) host memory");
                }
            }
            e = static_scratch_setup(cfg->device);  // address of this GPU's static scratch, its staging buffer
            if (e != hipSuccess) {
                int rc = hip_fail(nullptr, e, "static scratch set-up");
                delete s;
                return rc;
            }
            std::vector<float2> cs;
            build_cos_sin(s->inv_freq, cfg->max_positions, cs);
            e = hipMalloc((void **)&s->cs_dev, cs.size() * sizeof(float2));
            if (e == hipSuccess) e = hipMemcpy(s->cs_dev, cs.data(), cs.size() * sizeof(float2), hipMemcpyHostToDevice);
        }
        if (e != hipSuccess) {
            int rc = hip_fail(nullptr, e, "store create");
            if (s->cs_dev) (void)hipFree(s->cs_dev);
            delete s;
            return rc;
        }
    }
    *out = s;
    return KVP_OK;
}

int kvp_store_destroy(kvp_store_t *s)
{
    if (!s) return KVP_E_INVAL;
    if (!s->dry) {
        (void)hipSetDevice(s->cfg.device);
        bool unsettled = false;  // launches from kept plans that no event of ours stands behind
        for (auto &e : s->pf_set) unsettled |= e.used_since_event;
        for (auto &e : s->pk_set) unsettled |= e.used_since_event;
        unsettled |= s->ring.unsettled();
        if (s->cfg.device < MAX_DEVICES) {
            kvp_store::PrefillCached &se = g_static[s->cfg.device].entry;
            if (se.owner == s->serial) {  // the scratch holds a plan of this store: forget it
                unsettled |= se.used_since_event;
                se.used_since_event = false;
                se.valid = false;
                se.owner = 0;
            }
        }
        if (unsettled) (void)hipDeviceSynchronize();
        s->ring.release();
        for (auto &e : s->pf_set) e.own.release(false);
        for (auto &e : s->pk_set) e.own.release(false);
        if (s->cs_dev) (void)hipFree(s->cs_dev);
    } else {
        s->ring.release();
        for (auto &e : s->pf_set) e.own.release(true);
        for (auto &e : s->pk_set) e.own.release(true);
    }
    delete s;
    return KVP_OK;
}

}  // extern "C"

namespace {

// Copies K, V [n_layers][n_kv_heads][rows][head_dim] into a new blob of the arena.
int put_blob(kvp_store *s, int rows, const void *k, const void *v, int src_on_device, void *hip_stream, PacketRec &rec)
{
    const kvp_config_t &g = s->cfg;
    const uint64_t row_bytes = (uint64_t)g.head_dim * s->esize;
    // (layer, head) slices follow each other without padding: skewing equal-length packets by a
    // few rows per slice or per blob was measured and changed nothing
    const int stride = rows;
    const uint64_t n_slices = (uint64_t)g.n_layers * g.n_kv_heads;
    const uint64_t half_bytes = n_slices * stride * row_bytes;
    const uint64_t need = align_up(2 * half_bytes);
    if (s->used_bytes + need > g.arena_bytes)
        return fail(s, KVP_E_NOSPACE, "arena full: %llu used + %llu needed > %llu", (unsigned long long)s->used_bytes,
                    (unsigned long long)need, (unsigned long long)g.arena_bytes);
    if (!s->dry) {
        HIP_TRY(s, hipSetDevice(g.device));
        char *dst = (char *)g.arena + s->used_bytes;
        hipMemcpyKind kind = s->arena_host ? hipMemcpyDefault : src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
        hipStream_t st = (hipStream_t)hip_stream;
        const uint64_t slice_bytes = (uint64_t)rows * row_bytes;
        HIP_TRY(s, hipMemcpy2DAsync(dst, stride * row_bytes, k, slice_bytes, slice_bytes, n_slices, kind, st));
        HIP_TRY(s, hipMemcpy2DAsync(dst + half_bytes, stride * row_bytes, v, slice_bytes, slice_bytes, n_slices, kind, st));
        if (!src_on_device) HIP_TRY(s, hipStreamSynchronize(st));  // host buffers may be reused on return
    }
    rec.elem_off = (int64_t)(s->used_bytes / s->esize);
    rec.stride = stride;
    s->used_bytes += need;
    return KVP_OK;
}

}  // namespace

extern "C" {

int kvp_store_put(kvp_store_t *s, int64_t packet_id, int32_t n_tokens, const void *k, const void *v,
                  int32_t src_on_device, void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    if (packet_id < 0) return fail(s, KVP_E_INVAL, "packet id %lld < 0", (long long)packet_id);
    if (n_tokens < 1) return fail(s, KVP_E_INVAL, "n_tokens %d < 1", n_tokens);
    if (!s->dry && (!k || !v)) return fail(s, KVP_E_INVAL, "k or v is null");
    if (s->dir.count(packet_id)) return fail(s, KVP_E_EXISTS, "packet %lld already stored", (long long)packet_id);
    PacketRec rec;
    rec.n_tokens = n_tokens;
    int rc = put_blob(s, n_tokens, k, v, src_on_device, hip_stream, rec);
    if (rc) return rc;
    s->dir[packet_id] = rec;
    return KVP_OK;
}

int kvp_store_put_header(kvp_store_t *s, const void *k, const void *v, int32_t src_on_device, void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    if (s->cfg.n_header < 1) return fail(s, KVP_E_INVAL, "the store was created with n_header = %d", s->cfg.n_header);
    if (!s->dry && (!k || !v)) return fail(s, KVP_E_INVAL, "k or v is null");
    if (s->header.n_tokens) return fail(s, KVP_E_EXISTS, "the header is already stored");
    PacketRec rec;
    int rc = put_blob(s, s->cfg.n_header, k, v, src_on_device, hip_stream, rec);
    if (rc) return rc;
    rec.n_tokens = s->cfg.n_header;
    s->header = rec;
    return KVP_OK;
}

int kvp_store_put_body(kvp_store_t *s, int64_t packet_id, int32_t n_tokens, const void *k, const void *v,
                       int32_t src_on_device, void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    if (packet_id < 0) return fail(s, KVP_E_INVAL, "packet id %lld < 0", (long long)packet_id);
    if (!s->header.n_tokens) return fail(s, KVP_E_INVAL, "no header stored (kvp_store_put_header)");
    if (n_tokens <= s->cfg.n_header) return fail(s, KVP_E_INVAL, "n_tokens %d does not exceed the %d header rows", n_tokens, s->cfg.n_header);
    if (!s->dry && (!k || !v)) return fail(s, KVP_E_INVAL, "k or v is null");
    if (s->dir.count(packet_id)) return fail(s, KVP_E_EXISTS, "packet %lld already stored", (long long)packet_id);
    PacketRec rec;
    rec.n_tokens = n_tokens;
    rec.head_rows = s->cfg.n_header;
    int rc = put_blob(s, n_tokens - s->cfg.n_header, k, v, src_on_device, hip_stream, rec);
    if (rc) return rc;
    s->dir[packet_id] = rec;
    return KVP_OK;
}

int32_t kvp_store_packet_len(const kvp_store_t *s, int64_t packet_id)
{
    if (!s) return KVP_E_INVAL;
    auto it = s->dir.find(packet_id);
    return it == s->dir.end() ? KVP_E_NOTFOUND : it->second.n_tokens;
}

int32_t kvp_store_packet_rows(const kvp_store_t *s, int64_t packet_id, int32_t layer)
{
    if (!s || layer < 0 || layer >= s->cfg.n_layers) return KVP_E_INVAL;
    auto it = s->dir.find(packet_id);
    if (it == s->dir.end()) return KVP_E_NOTFOUND;
    return it->second.compressed() ? it->second.rows[layer] : it->second.n_tokens;
}

int kvp_store_put_compressed(kvp_store_t *s, int64_t packet_id, int32_t span, const int32_t *n_rows,
                             const void *k, const void *v, int32_t src_on_device, void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    if (packet_id < 0) return fail(s, KVP_E_INVAL, "packet id %lld < 0", (long long)packet_id);
    if (span < 1) return fail(s, KVP_E_INVAL, "span %d < 1", span);
    if (!n_rows) return fail(s, KVP_E_INVAL, "n_rows is null");
    if (s->dir.count(packet_id)) return fail(s, KVP_E_EXISTS, "packet %lld already stored", (long long)packet_id);
    const kvp_config_t &g = s->cfg;
    const uint64_t row_bytes = (uint64_t)g.head_dim * s->esize;
    PacketRec rec;
    rec.elem_off = (int64_t)(s->used_bytes / s->esize);
    rec.n_tokens = rec.stride = span;
    uint64_t total_rows = 0;
    for (int l = 0; l < g.n_layers; ++l) {
        if (n_rows[l] < 0 || n_rows[l] > span) return fail(s, KVP_E_INVAL, "layer %d keeps %d rows of a span of %d", l, n_rows[l], span);
        rec.rows.push_back(n_rows[l]);
        rec.layer_off.push_back(rec.elem_off + (int64_t)(2 * total_rows * g.n_kv_heads * g.head_dim));
        total_rows += (uint64_t)n_rows[l];
    }
    if (!s->dry && total_rows > 0 && (!k || !v)) return fail(s, KVP_E_INVAL, "k or v is null");
    const uint64_t need = align_up(std::max<uint64_t>(2 * total_rows * g.n_kv_heads * row_bytes, 1));
    if (s->used_bytes + need > g.arena_bytes)
        return fail(s, KVP_E_NOSPACE, "arena full: %llu used + %llu needed > %llu", (unsigned long long)s->used_bytes,
                    (unsigned long long)need, (unsigned long long)g.arena_bytes);
    if (!s->dry) {
        HIP_TRY(s, hipSetDevice(g.device));
        hipMemcpyKind kind = s->arena_host ? hipMemcpyDefault : src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
        hipStream_t st = (hipStream_t)hip_stream;
        uint64_t src_off = 0;
        for (int l = 0; l < g.n_layers; ++l) {
            const uint64_t part = (uint64_t)n_rows[l] * g.n_kv_heads * row_bytes;  // K (or V) of this layer
            if (!part) continue;
            char *dst = (char *)g.arena + (uint64_t)rec.layer_off[l] * s->esize;
            HIP_TRY(s, hipMemcpyAsync(dst, (const char *)k + src_off, part, kind, st));
            HIP_TRY(s, hipMemcpyAsync(dst + part, (const char *)v + src_off, part, kind, st));
            src_off += part;
        }
        if (!src_on_device) HIP_TRY(s, hipStreamSynchronize(st));
    }
    s->dir[packet_id] = rec;
    s->used_bytes += need;
    return KVP_OK;
}

uint64_t kvp_store_bytes_used(const kvp_store_t *s) { return s ? s->used_bytes : 0; }

int32_t kvp_store_arena_on_host(const kvp_store_t *s) { return s ? (s->arena_host ? 1 : 0) : KVP_E_INVAL; }

// -------------------------------------------------------------------------------------
int kvp_assemble(kvp_store_t *s, const kvp_request_t *reqs, int32_t n_req, int32_t layer_begin,
                 int32_t layer_end, kvp_cache_t *cache, void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    const kvp_config_t &g = s->cfg;
    if (n_req < 0 || (n_req > 0 && !reqs)) return fail(s, KVP_E_INVAL, "bad request list");
    if (layer_begin < 0 || layer_end > g.n_layers || layer_begin > layer_end)
        return fail(s, KVP_E_INVAL, "layer range [%d, %d) outside [0, %d]", layer_begin, layer_end, g.n_layers);
    CacheCheck cc;
    int rc = check_cache(s, cache, n_req, cc);
    if (rc) return rc;

    // A request that names a compressed packet (Sec. 5.4) takes the layer-by-layer route: its
    // layers have different row counts.
    for (int r = 0; r < n_req; ++r) {
        const kvp_request_t &q = reqs[r];
        if (q.k < 0 || (q.k > 0 && !q.packet_ids)) return fail(s, KVP_E_INVAL, "request %d: bad packet list", r);
        for (int j = 0; j < q.k; ++j) {
            auto it = s->dir.find(q.packet_ids[j]);
            if (it != s->dir.end() && it->second.compressed())
                return assemble_compressed(s, reqs, n_req, layer_begin, layer_end, cache, cc, hip_stream);
        }
    }

    // offsets Delta_j (Sec. 4.2.1 step 4: realign, then concatenate): one segment per packet
    const int tile_rows = tile_rows_for(s, cache);
    std::vector<AsmSeg> segs;
    int64_t n_tiles = 0, rows_total = 0, rows_unique = 0;
    std::unordered_set<int64_t> seen;
    std::vector<int> ctx(n_req), first_blk(n_req, 0), n_blk(n_req, 0);
    for (int r = 0; r < n_req; ++r) {
        const kvp_request_t &q = reqs[r];
        if (q.base_pos < 0) return fail(s, KVP_E_INVAL, "request %d: base_pos %d < 0", r, q.base_pos);
        int64_t pos = q.base_pos;
        for (int j = 0; j < q.k; ++j) {
            auto it = s->dir.find(q.packet_ids[j]);
            if (it == s->dir.end()) return fail(s, KVP_E_NOTFOUND, "request %d: packet %lld not in the store", r, (long long)q.packet_ids[j]);
            const PacketRec &p = it->second;
            rows_total += p.n_tokens;
            if (seen.insert(q.packet_ids[j]).second) rows_unique += p.n_tokens;
            if (pos + p.n_tokens > g.max_positions)
                return fail(s, KVP_E_CAPACITY, "request %d: context exceeds max_positions %d", r, g.max_positions);
            if (p.head_rows) {  // the header rows come from the shared copy, at the packet's own Delta
                segs.push_back(AsmSeg{s->header.elem_off, s->header.stride, p.head_rows, (int32_t)pos, (int32_t)pos, r, 0, (int32_t)n_tiles, 0});
                n_tiles += tiles_of(p.head_rows, tile_rows);
            }
            segs.push_back(AsmSeg{p.elem_off, p.stride, p.body_rows(), (int32_t)pos + p.head_rows, (int32_t)pos, r, 0, (int32_t)n_tiles, 0});
            n_tiles += tiles_of(p.body_rows(), tile_rows);
            pos += p.n_tokens;
        }
        if (pos > cc.cap_rows) return fail(s, KVP_E_CAPACITY, "request %d: %lld rows do not fit the cache (%lld)", r, (long long)pos, (long long)cc.cap_rows);
        ctx[r] = (int)pos;
        if (cache->layout == KVP_PAGED && pos > q.base_pos) {
            first_blk[r] = q.base_pos >> cc.shift;
            n_blk[r] = (int)((pos - 1) >> cc.shift) + 1;
        }
    }
    rc = run_gather(s, segs, n_tiles, tile_rows, false, layer_begin, layer_end - layer_begin, cache, cc, n_req, first_blk, n_blk,
                    gather_streams_once(s, rows_total, rows_unique, layer_end - layer_begin), hip_stream);
    if (rc) return rc;
    for (int r = 0; r < n_req; ++r) {
        cache->ctx_len[r] = ctx[r];
        if (cache->ctx_rows)
            for (int l = layer_begin; l < layer_end; ++l) cache->ctx_rows[(int64_t)r * g.n_layers + l] = ctx[r];
    }
    return KVP_OK;
}

// -------------------------------------------------------------------------------------
}  // extern "C"

namespace {

// Partial slots: group gi owns slots gi * stride .. + stride - 1 (stride = the largest split
// count of the call), so the combine kernel knows where a group's partials are before it has
// read the group's record.  stride 0: nothing is split, no slots.
void assign_part_slots(std::vector<AttnGroup> &groups, std::vector<AttnItem> &items, int stride, int &n_slots)
{
    for (size_t gi = 0; gi < groups.size(); ++gi) groups[gi].part0 = (int32_t)gi * stride;
    for (auto &it : items)
        if (it.part_slot >= 0) it.part_slot += groups[it.group].part0;
    n_slots = (int)groups.size() * stride;
}

// Workgroups are dealt to the 8 XCDs round-robin by index, and each XCD has its own L2.
// Items that read the same K/V rows (same request, KV head and kv range, different row
// blocks) are therefore placed 8 apart, next to each other in launch order: they run on
// one XCD at about the same time and all but the first find the tiles in its L2.  Cohorts
// of unequal size are padded with null items (n_rows = 0: the workgroup exits at once).
// Cohorts go out longest first (kv rows x query rows of their largest member): workgroups
// start in index order as compute units fall free, so the long items of a ragged batch start
// early and the short ones fill the end of the launch.
bool xcd_order(std::vector<AttnItem> &items)  // returns whether any two items share their K/V rows
{
    constexpr int XCDS = 8;
    const int n = (int)items.size();
    // items by cohort key, original order inside a cohort
    struct Ref { int64_t key; int idx; };
    std::vector<Ref> refs(n);
    for (int i = 0; i < n; ++i) {
        const AttnItem &it = items[i];
        refs[i] = Ref{((int64_t)it.req << 40) ^ ((int64_t)it.kv_head << 28) ^ (int64_t)it.split, i};
    }
    std::sort(refs.begin(), refs.end(), [](const Ref &x, const Ref &y) { return x.key != y.key ? x.key < y.key : x.idx < y.idx; });
    struct Cohort { int first, count, order; int64_t work; };  // refs[first .. first + count); order = its first item's index
    std::vector<Cohort> cohorts;
    bool shared = false;
    for (int i = 0; i < n;) {
        int j = i;
        int64_t work = 0;
        for (; j < n && refs[j].key == refs[i].key; ++j) {
            const AttnItem &it = items[refs[j].idx];
            work = std::max(work, (int64_t)(it.kv_end - it.kv_begin) * it.n_rows);
        }
        cohorts.push_back(Cohort{i, j - i, refs[i].idx, work});
        shared |= j - i > 1;
        i = j;
    }
    // longest first; equal work keeps the planner's order
    std::sort(cohorts.begin(), cohorts.end(),
              [](const Cohort &x, const Cohort &y) { return x.work != y.work ? x.work > y.work : x.order < y.order; });
    std::vector<AttnItem> out;
    out.reserve(items.size() + 64);
    if (!shared) {
        for (const Cohort &c : cohorts) out.push_back(items[refs[c.first].idx]);
        items.swap(out);
        return false;
    }
    AttnItem null_item{};
    null_item.group = -1;
    for (size_t c0 = 0; c0 < cohorts.size(); c0 += XCDS) {
        const size_t c1 = std::min(cohorts.size(), c0 + XCDS);
        int depth = 0;
        for (size_t c = c0; c < c1; ++c) depth = std::max(depth, cohorts[c].count);
        const bool last_block = c1 == cohorts.size();
        for (int j = 0; j < depth; ++j)
            for (size_t c = c0; c < c0 + XCDS; ++c) {
                if (c < c1 && j < cohorts[c].count) out.push_back(items[refs[cohorts[c].first + j].idx]);
                else if (!(last_block && c >= c1 && j + 1 == depth)) out.push_back(null_item);
            }
    }
    while (!out.empty() && out.back().group < 0) out.pop_back();
    items.swap(out);
    return true;
}

// The kept plan with this signature on this stream (hit), or the entry a new plan would be built
// in: a fresh one while the set may grow, else an invalid one, else the least recently used.
// Nothing of the victim is changed here: the caller invalidates it only once the new plan has
// passed every check, so a call that fails leaves the kept plans as they were.
constexpr int MAX_CAPTURED_PLANS = 64;  // plans a HIP graph launches from, per entry point and store

kvp_store::PrefillCached *find_plan(kvp_store *s, std::deque<kvp_store::PrefillCached> &set, const std::vector<int32_t> &sig,
                                    void *stream, uint64_t &sig_hash, bool &hit)
{
    sig_hash = 1469598103934665603ull;
    for (int32_t x : sig) sig_hash = (sig_hash ^ (uint32_t)x) * 1099511628211ull;
    kvp_store::PrefillCached *victim = nullptr;
    int replaceable = 0;
    for (auto &e : set) {
        if (e.valid && e.sig_hash == sig_hash && e.stream == stream && e.sig == sig) {
            hit = true;
            e.last_use = ++s->pf_clock;
            return &e;
        }
        if (e.captured) continue;  // a graph launches from it
        ++replaceable;
        if (!victim || (!e.valid && victim->valid) || (e.valid == victim->valid && e.last_use < victim->last_use)) victim = &e;
    }
    hit = false;
    if (!victim || (victim->valid && replaceable < std::max(PlanRing::SLOTS, s->cfg.n_layers + 1))) {
        set.emplace_back();  // (an empty entry: nothing is lost if the call fails later)
        victim = &set.back();
    }
    return victim;
}

int captured_plans(const std::deque<kvp_store::PrefillCached> &set)
{
    int n = 0;
    for (const auto &e : set) n += e.captured ? 1 : 0;
    return n;
}

// Block ids of the table rows a call will read, checked before anything is changed.
int check_block_table(kvp_store *s, const kvp_cache_t *c, int n_req, const std::vector<int> &first_blk, const std::vector<int> &n_blk)
{
    if (c->layout != KVP_PAGED) return KVP_OK;
    for (int r = 0; r < n_req; ++r) {
        const int32_t *row = c->block_table + (int64_t)r * c->max_blocks_per_req;
        for (int b = first_blk[r]; b < n_blk[r]; ++b)
            if (row[b] < 0 || row[b] >= c->n_blocks)
                return fail(s, KVP_E_INVAL, "block_table[%d][%d] = %d is outside [0, %d)", r, b, row[b], c->n_blocks);
    }
    return KVP_OK;
}

// Before an entry's plan buffer is rewritten: if launches newer than the entry's event may
// still read it, put an event behind them now (the buffer's ensure() then waits for it).
int settle_plan_entry(kvp_store *s, kvp_store::PrefillCached &e)
{
    if (s->dry || !e.used_since_event) return KVP_OK;
    e.used_since_event = false;
    PlanSlot &slot = e.own;
    hipError_t rc = slot.ev ? hipEventRecord(slot.ev, (hipStream_t)e.stream) : hipErrorInvalidHandle;
    if (rc == hipSuccess) {
        slot.pending = true;
        return KVP_OK;
    }
    (void)hipGetLastError();  // (the stream may be gone: wait for the whole device instead)
    HIP_TRY(s, hipDeviceSynchronize());
    slot.pending = false;
    return KVP_OK;
}

struct PrefillPlan {
    int kind = ATTN_GENERIC, bm = 8, bn = 64;
    std::vector<ReqMeta> reqs;
    std::vector<int32_t> row_req;
    std::vector<AttnGroup> groups;
    std::vector<AttnItem> items;
    int n_slots = 0, part_stride = 1, max_group_rows = 0;
    bool any_split = false;
    bool mixed = false;  // MFMA kernel, 256-row blocks: some groups are half blocks
    bool split_in_wg = false;  // MFMA kernel, 128-row blocks: 8 waves in two groups on alternate tiles
    bool shared_rows = false;  // some work items read the same K/V rows (several row blocks per request and head),
                               // or the launch is short: either way no streaming hint on the tile loads
    int split_len0 = 0;        // kv rows per split of request 0
};

constexpr int MFMA_BM = 128;
constexpr int GENERIC_BM = 8;
constexpr int MAX_SPLITS = 64;

// Many tiles per compute unit to stream with 128-row blocks (long contexts, few query rows:
// HBM-bound): such launches take one 8-wave workgroup per CU whose two wave groups work on
// alternate tiles, four tile stages deep -- bytes in flight are what counts there (measured on 8
// requests of 16.9K context: 32 query rows 158 us with 192 four-wave items, 133 us with 512,
// 126 us this way; one query row 119 -> 111 us).
bool streams_many_tiles(const kvp_store *s, int64_t tiles, int bm)
{
    return bm == 128 && tiles >= 16 * (int64_t)s->n_cu;
}

// Work items a launch should have.  Three quarters of the CU count when the call reads little
// (one 8K request: every extra split costs partial traffic and the items are latency-bound
// anyway); one per CU for the streaming shape above.
int target_items(const kvp_store *s, int64_t tiles = 0, int bm = 0)
{
    if (s->target_items > 0) return s->target_items;
    if (streams_many_tiles(s, tiles, bm)) return s->n_cu;
    return s->n_cu * 3 / 4;
}

// Groups of packed rows and their split-KV items.  Every group of a request gets the same
// split length (a multiple of bn rows), chosen so the launch has about target_items work
// items; a group's kv range stops at the last row any of its query rows may see.
bool use_mfma(const kvp_store *s, const kvp_cache_t *c)
{
    const kvp_config_t &g = s->cfg;
    if (g.dtype != KVP_BF16 || g.head_dim != 128 || s->force_generic) return false;
    return !(c && c->layout == KVP_PAGED && c->block_size < MFMA_MIN_BLOCK_SIZE);
}

void plan_prefill(const kvp_store *s, const kvp_cache_t *cache, int n_req, const int32_t *ctx_len, const int32_t *pos0, const int32_t *q_off,
                  PrefillPlan &p)
{
    const kvp_config_t &g = s->cfg;
    const int gq = g.n_q_heads / g.n_kv_heads;
    const bool mfma = use_mfma(s, cache);
    // paged + MFMA: an item's blocks must fit the kernel's LDS id table
    const int max_split = (mfma && cache->layout == KVP_PAGED)
                              ? (MFMA_MAX_ITEM_BLOCKS - 1) * cache->block_size / 64 * 64
                              : INT32_MAX;
    p.kind = mfma ? ATTN_MFMA : ATTN_GENERIC;
    p.bm = mfma ? MFMA_BM : GENERIC_BM;
    if (mfma) {  // row blocks of 256 when some request has that many packed rows
        for (int r = 0; r < n_req; ++r)
            if ((int64_t)(q_off[r + 1] - q_off[r]) * gq >= 2 * MFMA_BM) p.bm = 2 * MFMA_BM;
        if (s->force_bm == 128 || s->force_bm == 256) p.bm = s->force_bm;
    }
    const int min_split = mfma ? 256 : 64;
    p.reqs.resize(n_req);
    int64_t n_groups = 0;
    for (int r = 0; r < n_req; ++r) {
        int n_q = q_off[r + 1] - q_off[r];
        p.reqs[r] = ReqMeta{ctx_len[r], q_off[r], n_q, pos0[r]};
        for (int t = 0; t < n_q; ++t) p.row_req.push_back(r);
        n_groups += (int64_t)g.n_kv_heads * (((int64_t)n_q * gq + p.bm - 1) / p.bm);
    }
    if (n_groups == 0) return;
    int64_t tiles = 0;  // 64-row tiles all the items together will read
    for (int r = 0; r < n_req; ++r)
        tiles += (int64_t)g.n_kv_heads * (((int64_t)p.reqs[r].n_q * gq + p.bm - 1) / p.bm) * ((p.reqs[r].ctx_len + p.reqs[r].n_q + 63) / 64);
    int want = (int)std::min<int64_t>(MAX_SPLITS, (target_items(s, tiles, mfma ? p.bm : 0) + n_groups - 1) / n_groups);
    if (want < 1) want = 1;
    p.split_in_wg = mfma && streams_many_tiles(s, tiles, p.bm);
    for (int r = 0; r < n_req; ++r) {
        const ReqMeta &rq = p.reqs[r];
        if (rq.n_q == 0) continue;
        const int total = rq.ctx_len + rq.n_q;
        int split_len = (total + want - 1) / want;
        split_len = std::max(split_len, min_split);
        split_len = (split_len + p.bn - 1) / p.bn * p.bn;
        split_len = std::min(split_len, max_split);
        if (r == 0) p.split_len0 = split_len;
        const int M = rq.n_q * gq;
        for (int h = 0; h < g.n_kv_heads; ++h)
            for (int m0 = 0; m0 < M; m0 += p.bm) {
                AttnGroup gp;
                gp.req = r;
                gp.kv_head = h;
                gp.m0 = m0;
                gp.n_rows = std::min(p.bm, M - m0);
                // a block of 256 of which at most half is filled (the last rows of a request)
                // runs as a half block: same compute unit, half the time
                const bool half_block = mfma && p.bm == 2 * MFMA_BM && gp.n_rows <= MFMA_BM && s->mixed_blocks;
                if (half_block) p.mixed = true;
                const int t_last = (m0 + gp.n_rows - 1) / gq;
                const int vis = rq.ctx_len + t_last + 1;
                gp.n_splits = (vis + split_len - 1) / split_len;
                gp.part0 = 0;  // set below, once the slot stride is known
                gp.q_off = rq.q_off;
                gp.pad1 = 0;
                if (gp.n_splits > 1) {
                    p.any_split = true;
                    p.max_group_rows = std::max(p.max_group_rows, gp.n_rows);
                }
                p.part_stride = std::max(p.part_stride, gp.n_splits);
                for (int sp = 0; sp < gp.n_splits; ++sp) {
                    AttnItem it{};
                    it.group = (int)p.groups.size();
                    it.split = sp;
                    it.kv_begin = sp * split_len;
                    it.kv_end = std::min(vis, (sp + 1) * split_len);
                    it.half_block = half_block ? 1 : 0;
                    it.req = r;
                    it.kv_head = h;
                    it.m0 = m0;
                    it.n_rows = gp.n_rows;
                    it.ctx_len = rq.ctx_len;
                    it.pos0 = rq.pos0;
                    it.q_off = rq.q_off;
                    it.part_slot = gp.n_splits > 1 ? sp : -1;  // relative to the group until the stride is known
                    it.n_q = rq.n_q;
                    p.items.push_back(it);
                }
                p.groups.push_back(gp);
            }
    }
    assign_part_slots(p.groups, p.items, p.any_split ? p.part_stride : 0, p.n_slots);
    p.shared_rows = xcd_order(p.items) || tiles < 16 * (int64_t)s->n_cu;  // (short launches: the hint measured slower)
}

// The items of a one-request MFMA launch as a formula in the kernel arguments (AttnInline), if
// the launch is that regular: rebuilding every item with the kernel's own function must give
// exactly the planned item; else t.n = 0.
void fill_inline_items(const kvp_store *s, int n_req, const ReqMeta *reqs, const std::vector<AttnGroup> &groups,
                       const std::vector<AttnItem> &items, int bm, int part_stride, int split_len, int gq, AttnInline &t)
{
    t.n = 0;
    const int n_kv = s->cfg.n_kv_heads;
    if (!s->inline_items || n_req != 1 || (int)groups.size() != n_kv || items.empty() || split_len <= 0 || reqs[0].q_off != 0 ||
        reqs[0].n_q * gq > bm)
        return;
    t.ctx_len = reqs[0].ctx_len;
    t.pos0 = reqs[0].pos0;
    t.n_q = reqs[0].n_q;
    t.n_rows = reqs[0].n_q * gq;
    t.split_len = split_len;
    t.ns = groups[0].n_splits;
    t.vis = 0;
    for (const AttnItem &it : items) t.vis = std::max(t.vis, it.kv_end);
    if ((int64_t)n_kv * t.ns != (int64_t)items.size()) return;
    for (int n_front : {t.ns, t.ns - 1}) {  // the last splits in place, or behind all the others
        if (n_front < 1 && t.ns > 1) continue;
        t.n_front = n_front;
        bool same = true;
        for (size_t i = 0; i < items.size() && same; ++i) {
            const AttnItem &want = items[i];
            const AttnItem got = attn_inline_item(t, (int)i, n_kv, part_stride);
            same = got.group == want.group && got.split == want.split && got.kv_begin == want.kv_begin && got.kv_end == want.kv_end &&
                   got.req == want.req && got.kv_head == want.kv_head && got.m0 == want.m0 && got.n_rows == want.n_rows &&
                   got.ctx_len == want.ctx_len && got.q_off == want.q_off && got.part_slot == want.part_slot && got.n_q == want.n_q &&
                   got.pos0 == want.pos0 && got.half_block == want.half_block;
        }
        if (same) {
            t.n = (int32_t)items.size();
            return;
        }
    }
}

uint64_t q_rot_bytes(const kvp_store *s, int64_t tot_q)
{
    return align_up((uint64_t)tot_q * s->cfg.n_q_heads * s->cfg.head_dim * s->esize);
}

}  // namespace

extern "C" {

uint64_t kvp_prefill_workspace_bytes(const kvp_store_t *s, int32_t n_req, int32_t max_tot_q, int32_t max_ctx)
{
    if (!s || n_req < 0 || max_tot_q < 0 || max_ctx < 0) return 0;
    const kvp_config_t &g = s->cfg;
    const int gq = g.n_q_heads / g.n_kv_heads;
    const bool mfma = use_mfma(s, nullptr);
    const int bm = mfma ? MFMA_BM : GENERIC_BM;  // smaller or larger row blocks need no more
    // groups <= Hkv * (rows / bm + one ragged block per request); every group has at most
    // ceil(target / groups) <= target / groups + 1 splits (and never more than MAX_SPLITS)
    const uint64_t groups = (uint64_t)g.n_kv_heads * ((uint64_t)max_tot_q * gq / bm + (uint64_t)n_req);
    // (a paged cache may force extra splits: at most max_ctx / 32704 more per group)
    const uint64_t extra = (uint64_t)max_ctx / ((MFMA_MAX_ITEM_BLOCKS - 1) * MFMA_MIN_BLOCK_SIZE / 64 * 64);
    const uint64_t slots = (uint64_t)std::max(target_items(s), 2 * s->n_cu) + (2 + extra) * groups;
    // (the MFMA kernel may pick 256-row blocks: twice the rows per slot, no more slots)
    return q_rot_bytes(s, max_tot_q) + slots * (mfma ? 2 * bm : bm) * (g.head_dim + 2) * sizeof(float) + ALIGN;
}

}  // extern "C"

namespace {

// kvp_query_prefill and kvp_query_prefill_static.  `fixed`: the static scratch's plan entry (the
// plan then lives in the scratch, which the call neither allocates nor frees), or nullptr: the
// plan goes into one of the store's kept entries, each with a buffer of its own.
int query_prefill_impl(kvp_store *s, kvp_cache_t *cache, int32_t layer, const void *q, const void *k_new,
                       const void *v_new, const int32_t *q_offsets, int32_t n_req, uint32_t flags, void *workspace,
                       uint64_t workspace_bytes, void *out, void *hip_stream, kvp_store::PrefillCached *fixed)
{
    const kvp_config_t &g = s->cfg;
    if (n_req < 0 || !q_offsets) return fail(s, KVP_E_INVAL, "bad request count or q_offsets is null");
    if (layer < 0 || layer >= g.n_layers) return fail(s, KVP_E_INVAL, "layer %d outside [0, %d)", layer, g.n_layers);
    if (flags & ~KVP_PREROTATED) return fail(s, KVP_E_INVAL, "unknown flags 0x%x", flags);
    CacheCheck cc;
    int rc = check_cache(s, cache, n_req, cc);
    if (rc) return rc;
    if (q_offsets[0] != 0) return fail(s, KVP_E_INVAL, "q_offsets[0] must be 0");
    std::vector<int> first_blk(n_req, 0), n_blk(n_req, 0);
    std::vector<int32_t> rows(n_req, 0);  // rows of this layer per request (= ctx_len without compressed packets)
    for (int r = 0; r < n_req; ++r) {
        int n_q = q_offsets[r + 1] - q_offsets[r];
        if (n_q < 0) return fail(s, KVP_E_INVAL, "q_offsets is not non-decreasing at %d", r);
        const int pos = cache->ctx_len[r];  // position of the first query token
        const int c = cache->ctx_rows ? cache->ctx_rows[(int64_t)r * g.n_layers + layer] : pos;  // rows of this layer
        if (pos < 0) return fail(s, KVP_E_INVAL, "request %d: ctx_len %d < 0", r, pos);
        if (c < 0 || c > pos) return fail(s, KVP_E_INVAL, "request %d: ctx_rows %d outside [0, ctx_len %d]", r, c, pos);
        rows[r] = c;
        int64_t total = (int64_t)c + n_q;
        if ((int64_t)pos + n_q > g.max_positions) return fail(s, KVP_E_CAPACITY, "request %d: %lld positions exceed max_positions %d", r, (long long)pos + n_q, g.max_positions);
        if (total > cc.cap_rows) return fail(s, KVP_E_CAPACITY, "request %d: %lld rows do not fit the cache (%lld)", r, (long long)total, (long long)cc.cap_rows);
        if (cache->layout == KVP_PAGED && n_q > 0) n_blk[r] = (int)((total - 1) >> cc.shift) + 1;
    }
    const int tot_q = q_offsets[n_req];
    if (tot_q > 0 && !s->dry) {
        if (!q || !k_new || !v_new || !out) return fail(s, KVP_E_INVAL, "q, k_new, v_new or out is null");
        if (((uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)out) & 15)
            return fail(s, KVP_E_INVAL, "q, k_new, v_new, out must be 16-byte aligned");
    }

    int bt_stride = 0;
    for (int r = 0; r < n_req; ++r) bt_stride = std::max(bt_stride, n_blk[r]);

    // geometry signature: everything the plan is a function of
    std::vector<int32_t> &sig = s->sig_scratch;
    sig.clear();
    sig.push_back(cache->layout);
    sig.push_back(n_req);
    sig.push_back(cache->layout == KVP_CONTIG ? cache->t_cap : cache->block_size);
    sig.push_back(cache->layout == KVP_CONTIG ? 0 : cache->n_blocks);
    for (int r = 0; r < n_req; ++r) sig.push_back(cache->ctx_len[r]);
    for (int r = 0; r < n_req; ++r) sig.push_back(rows[r]);
    for (int r = 0; r <= n_req; ++r) sig.push_back(q_offsets[r]);
    if (cache->layout == KVP_PAGED)
        for (int r = 0; r < n_req; ++r) {
            const int32_t *row = cache->block_table + (int64_t)r * cache->max_blocks_per_req;
            sig.insert(sig.end(), row, row + n_blk[r]);
        }
    uint64_t sig_hash = 0;
    bool hit = false;
    if (!s->dry) HIP_TRY(s, hipSetDevice(g.device));
    const bool in_capture = capturing(s, hip_stream);
    if (in_capture && tot_q == 0) return KVP_OK;  // nothing to launch, and no plan to touch
    kvp_store::PrefillCached *found;
    if (fixed) {
        found = fixed;
        sig_hash = 0;
        hit = fixed->valid && fixed->owner == s->serial && fixed->stream == hip_stream && fixed->sig == sig;
    } else {
        found = find_plan(s, s->pf_set, sig, hip_stream, sig_hash, hit);
    }
    kvp_store::PrefillCached &pf = *found;
    const uint64_t qrb = use_mfma(s, cache) ? 0 : q_rot_bytes(s, tot_q);  // (the MFMA kernel rotates the query in registers)
    if (in_capture && !hit)
        return fail(s, KVP_E_INVAL, "kvp_query_prefill under stream capture needs the plan of an earlier call with the same "
                                    "geometry on the same stream (call it once before capturing)");
    if (in_capture && !pf.captured && captured_plans(s->pf_set) >= MAX_CAPTURED_PLANS)
        return fail(s, KVP_E_CAPACITY, "%d plans of this store are already held for HIP graphs (kvp_release_captured_plans)", MAX_CAPTURED_PLANS);

    if (!hit) {
        PrefillPlan p;
        plan_prefill(s, cache, n_req, rows.data(), cache->ctx_len, q_offsets, p);
        // (the MFMA kernel's partial rows are fp16: half the bytes of the generic kernel's)
        const uint64_t need = qrb + (uint64_t)p.n_slots * (uint64_t)part_slot_bytes(p.bm, g.head_dim, p.kind == ATTN_MFMA ? 1 : 0);
        const uint64_t bytes = p.reqs.size() * sizeof(ReqMeta) + p.row_req.size() * 4 + p.groups.size() * sizeof(AttnGroup) +
                               p.items.size() * sizeof(AttnItem) + (uint64_t)n_req * bt_stride * 4 + 6 * 64;
        // every check comes before the entry is touched: a call that fails has changed nothing
        if (tot_q > 0) {
            if (!s->dry && !workspace) return fail(s, KVP_E_INVAL, "workspace is null");
            if ((uintptr_t)workspace & (ALIGN - 1)) return fail(s, KVP_E_INVAL, "workspace must be 256-byte aligned");
            if (workspace_bytes < need)
                return fail(s, KVP_E_CAPACITY, fixed ? "this call needs %2$llu bytes of workspace, the static scratch holds %1$llu"
                                                     : "workspace too small: %llu < %llu",
                            (unsigned long long)workspace_bytes, (unsigned long long)need);
        }
        rc = check_block_table(s, cache, n_req, first_blk, n_blk);
        if (rc) return rc;
        AttnInline inl;
        inl.n = 0;
        if (p.kind == ATTN_MFMA)
            fill_inline_items(s, n_req, p.reqs.data(), p.groups, p.items, p.bm, p.part_stride, p.split_len0,
                              g.n_q_heads / g.n_kv_heads, inl);
        if (fixed && bytes > KVP_STATIC_PLAN_BYTES)
            return fail(s, KVP_E_CAPACITY, "the plan of this call (%llu bytes) exceeds the %llu the static scratch keeps for it",
                        (unsigned long long)bytes, (unsigned long long)KVP_STATIC_PLAN_BYTES);
        pf.valid = false;  // the entry's buffer is rewritten below
        pf.last_use = ++s->pf_clock;
        pf.owner = s->serial;
        PlanSlot *slot = &pf.own;
        rc = settle_plan_entry(s, pf);
        if (rc) return rc;
        int hrc = slot->ensure(bytes, s->dry);
        if (hrc) return hip_fail(s, (hipError_t)hrc, "plan buffer");
        PlanWriter w{slot->host, s->dry ? nullptr : slot->dev};
        ReqMeta *rh = w.put<ReqMeta>(p.reqs.size(), &pf.reqs_dev);
        if (!p.reqs.empty()) memcpy(rh, p.reqs.data(), p.reqs.size() * sizeof(ReqMeta));
        int32_t *rr = w.put<int32_t>(p.row_req.size(), &pf.row_req_dev);
        if (!p.row_req.empty()) memcpy(rr, p.row_req.data(), p.row_req.size() * 4);
        AttnGroup *gh = w.put<AttnGroup>(p.groups.size(), &pf.groups_dev);
        if (!p.groups.empty()) memcpy(gh, p.groups.data(), p.groups.size() * sizeof(AttnGroup));
        AttnItem *ih = w.put<AttnItem>(p.items.size(), &pf.items_dev);
        if (!p.items.empty()) memcpy(ih, p.items.data(), p.items.size() * sizeof(AttnItem));
        pf.bt_dev = nullptr;
        if (cache->layout == KVP_PAGED && bt_stride > 0) {
            int32_t *bh = w.put<int32_t>((uint64_t)n_req * bt_stride, &pf.bt_dev);
            rc = compact_block_table(s, cache, n_req, first_blk, n_blk, bt_stride, bh);
            if (rc) return rc;
        }
        {
            kvp_store::DebugPlan &dp = s->dbg_plan;
            const int64_t head[6] = {p.kind, p.bm, (int64_t)p.groups.size(), (int64_t)p.items.size(), p.n_slots, (int64_t)need};
            memcpy(dp.head, head, sizeof head);
            dp.groups.swap(p.groups);  // (already copied into the plan buffer above)
            dp.items.swap(p.items);
            dp.tiles.clear();
            dp.has_tiles = false;
            dp.inl_n = inl.n;
        }
        pf.slot = slot;
        pf.kind = p.kind;
        pf.bm = p.bm;
        pf.n_items = (int)s->dbg_plan.head[3];  // (the vectors themselves have moved into dbg_plan)
        pf.n_groups = (int)s->dbg_plan.head[2];
        pf.bt_stride = bt_stride;
        pf.tot_q = tot_q;
        pf.any_split = p.any_split;
        pf.mixed = p.mixed;
        pf.split_in_wg = p.split_in_wg;
        pf.shared_rows = p.shared_rows;
        pf.part_stride = p.part_stride;
        pf.max_group_rows = p.max_group_rows;
        pf.need = need;
        pf.sig = sig;
        pf.sig_hash = sig_hash;
        pf.stream = hip_stream;
        pf.inl.n = inl.n;
        if (inl.n) pf.inl = inl;
        if (s->dry || tot_q == 0) return KVP_OK;
        rc = upload_plan(s, slot, w.off, hip_stream);
        if (rc) return rc;
        pf.valid = true;
    } else if (tot_q > 0) {
        if (!s->dry && !workspace) return fail(s, KVP_E_INVAL, "workspace is null");
        if ((uintptr_t)workspace & (ALIGN - 1)) return fail(s, KVP_E_INVAL, "workspace must be 256-byte aligned");
        if (workspace_bytes < pf.need)
            return fail(s, KVP_E_CAPACITY, "workspace too small: %llu < %llu", (unsigned long long)workspace_bytes, (unsigned long long)pf.need);
    }
    if (s->dry || tot_q == 0) return KVP_OK;

    hipStream_t st = (hipStream_t)hip_stream;
    CacheView view = make_view(s, cache, cc.shift, pf.bt_dev, pf.bt_stride);

    if (pf.kind != ATTN_MFMA) {  // the MFMA kernel does the query side itself
        AppendArgs ap;
        ap.q = q;
        ap.k_new = k_new;
        ap.v_new = v_new;
        ap.q_rot = workspace;
        ap.cs = s->cs_dev;
        ap.cache = view;
        ap.reqs = pf.reqs_dev;
        ap.row_req = pf.row_req_dev;
        ap.tot_q = tot_q;
        ap.layer = layer;
        ap.n_q_heads = g.n_q_heads;
        ap.n_kv = g.n_kv_heads;
        ap.d = g.head_dim;
        ap.prerotated = (flags & KVP_PREROTATED) ? 1 : 0;
        ap.q_scale = 1.f;
        int e = launch_append(g.dtype, ap, hip_stream);
        if (e) return hip_fail(s, (hipError_t)e, "append launch");
    }

    int e = 0;
    AttnArgs at;
    at.q_rot = workspace;
    at.q = q;
    at.k_new = k_new;
    at.v_new = v_new;
    at.cs = s->cs_dev;
    at.prerotated = (flags & KVP_PREROTATED) ? 1 : 0;
    at.tiles = nullptr;
    at.arena = nullptr;
    at.k_tail = nullptr;
    at.n_layers_total = g.n_layers;
    at.cache = view;
    at.reqs = pf.reqs_dev;
    at.groups = pf.groups_dev;
    at.items = pf.items_dev;
    at.partials = (float *)((char *)workspace + qrb);
    at.part_f16 = pf.kind == ATTN_MFMA ? 1 : 0;
    at.out = out;
    at.n_items = pf.n_items;
    at.n_groups = pf.n_groups;
    at.layer = layer;
    at.n_q_heads = g.n_q_heads;
    at.n_kv = g.n_kv_heads;
    at.d = g.head_dim;
    at.bm = pf.bm;
    at.split_in_wg = s->force_split_in_wg >= 0 ? s->force_split_in_wg : (pf.split_in_wg ? 1 : 0);
    at.mixed = pf.mixed ? 1 : 0;
    at.nt_loads = s->nt_loads >= 0 ? s->nt_loads : (pf.shared_rows ? 0 : 1);
    at.part_stride = pf.part_stride;
    at.max_group_rows = pf.max_group_rows;
    at.g = g.n_q_heads / g.n_kv_heads;
    at.scale_log2e = (float)(1.4426950408889634 / sqrt((double)g.head_dim));
    at.inl.n = pf.inl.n;
    if (pf.inl.n) at.inl = pf.inl;
    e = launch_attention(g.dtype, at, pf.kind, hip_stream);
    if (e) return hip_fail(s, (hipError_t)e, "attention launch");
    if (pf.any_split) {
        e = launch_combine(g.dtype, at, hip_stream);
        if (e) return hip_fail(s, (hipError_t)e, "combine launch");
    }
    if (in_capture) {
        if (!fixed) pf.captured = true;  // the graph reads this plan at every replay: keep it until the store goes
    } else if (hit) {
        pf.used_since_event = true;
    } else {
        HIP_TRY(s, hipEventRecord(pf.slot->ev, st));
        pf.slot->pending = true;
    }
    return KVP_OK;
}

}  // namespace

extern "C" {

int kvp_query_prefill(kvp_store_t *s, kvp_cache_t *cache, int32_t layer, const void *q, const void *k_new,
                      const void *v_new, const int32_t *q_offsets, int32_t n_req, uint32_t flags, void *workspace,
                      uint64_t workspace_bytes, void *out, void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    return query_prefill_impl(s, cache, layer, q, k_new, v_new, q_offsets, n_req, flags, workspace, workspace_bytes, out,
                              hip_stream, nullptr);
}

uint64_t kvp_static_workspace_bytes(void) { return KVP_STATIC_SCRATCH_BYTES - KVP_STATIC_PLAN_BYTES; }

int kvp_query_prefill_static(kvp_store_t *s, kvp_cache_t *cache, int32_t layer, const void *q, const void *k_new,
                             const void *v_new, const int32_t *q_offsets, int32_t n_req, uint32_t flags, void *out,
                             void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    if (s->dry) return fail(s, KVP_E_INVAL, "kvp_query_prefill_static needs a store on a GPU");
    const int dev = s->cfg.device;
    if (dev < 0 || dev >= MAX_DEVICES || !g_static[dev].ready) return fail(s, KVP_E_HIP, "no static scratch on device %d", dev);
    StaticScratch &ss = g_static[dev];
    // the workspace is the scratch behind the plan: never the array's name, always its device address
    return query_prefill_impl(s, cache, layer, q, k_new, v_new, q_offsets, n_req, flags, ss.ptr + KVP_STATIC_PLAN_BYTES,
                              KVP_STATIC_SCRATCH_BYTES - KVP_STATIC_PLAN_BYTES, out, hip_stream, &ss.entry);
}

// -------------------------------------------------------------------------------------
// Attention over the retrieved packets in place (no cache): the plan is a list of tiles of
// at most 64 rows, each inside one stored packet or inside the query rows.
int kvp_prefill_packets(kvp_store_t *s, const kvp_request_t *reqs, int32_t n_req, int32_t layer, const void *q,
                        const void *k_new, const void *v_new, const int32_t *q_offsets, uint32_t flags, void *k_tail,
                        void *workspace, uint64_t workspace_bytes, void *out, void *hip_stream)
{
    if (!s) return KVP_E_INVAL;
    const kvp_config_t &g = s->cfg;
    if (g.dtype != KVP_BF16 || g.head_dim != 128)
        return fail(s, KVP_E_INVAL, "kvp_prefill_packets needs a bf16 store with head_dim 128");
    if (n_req < 0 || !q_offsets || (n_req > 0 && !reqs)) return fail(s, KVP_E_INVAL, "bad request list or q_offsets is null");
    if (layer < 0 || layer >= g.n_layers) return fail(s, KVP_E_INVAL, "layer %d outside [0, %d)", layer, g.n_layers);
    if (flags & ~KVP_PREROTATED) return fail(s, KVP_E_INVAL, "unknown flags 0x%x", flags);
    if (q_offsets[0] != 0) return fail(s, KVP_E_INVAL, "q_offsets[0] must be 0");

    std::vector<int32_t> &sig = s->sig_scratch;
    sig.clear();
    sig.push_back(n_req);
    bool any_compressed = false;
    for (int r = 0; r < n_req; ++r) {
        const kvp_request_t &rq = reqs[r];
        if (rq.k < 0 || (rq.k > 0 && !rq.packet_ids)) return fail(s, KVP_E_INVAL, "request %d: bad packet list", r);
        if (rq.base_pos != 0) return fail(s, KVP_E_INVAL, "request %d: base_pos must be 0 without a cache", r);
        if (q_offsets[r + 1] < q_offsets[r]) return fail(s, KVP_E_INVAL, "q_offsets is not non-decreasing at %d", r);
        sig.push_back(rq.k);
        sig.push_back(q_offsets[r + 1]);
        for (int j = 0; j < rq.k; ++j) {
            sig.push_back((int32_t)(rq.packet_ids[j] & 0xFFFFFFFF));
            sig.push_back((int32_t)(rq.packet_ids[j] >> 32));
            auto itp = s->dir.find(rq.packet_ids[j]);
            if (itp == s->dir.end()) return fail(s, KVP_E_NOTFOUND, "request %d: packet %lld not in the store", r, (long long)rq.packet_ids[j]);
            any_compressed |= itp->second.compressed();
        }
    }
    sig.push_back(any_compressed ? layer : -1);  // compressed packets (Sec. 5.4): every layer has its own rows, hence its own tiles
    const int tot_q = q_offsets[n_req];
    if (tot_q > 0 && !s->dry) {
        if (!q || !k_new || !v_new || !out || !k_tail) return fail(s, KVP_E_INVAL, "q, k_new, v_new, k_tail or out is null");
        if (((uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)out | (uintptr_t)k_tail) & 15)
            return fail(s, KVP_E_INVAL, "q, k_new, v_new, k_tail, out must be 16-byte aligned");
    }
    uint64_t sig_hash = 0;
    bool hit = false;
    if (!s->dry) HIP_TRY(s, hipSetDevice(g.device));
    const bool in_capture = capturing(s, hip_stream);
    if (in_capture && tot_q == 0) return KVP_OK;  // nothing to launch, and no plan to touch
    kvp_store::PrefillCached &pk = *find_plan(s, s->pk_set, sig, hip_stream, sig_hash, hit);
    if (in_capture && !hit)
        return fail(s, KVP_E_INVAL, "kvp_prefill_packets under stream capture needs the plan of an earlier call with the same "
                                    "requests on the same stream (call it once before capturing)");
    if (in_capture && !pk.captured && captured_plans(s->pk_set) >= MAX_CAPTURED_PLANS)
        return fail(s, KVP_E_CAPACITY, "%d plans of this store are already held for HIP graphs (kvp_release_captured_plans)", MAX_CAPTURED_PLANS);

    if (!hit) {
        const int gq = g.n_q_heads / g.n_kv_heads;
        std::vector<AttnTile> tiles;
        std::vector<ReqMeta> metas(n_req);
        std::vector<int> tile_begin(n_req), n_pkt_tiles(n_req);
        std::vector<int> pkt_tiles(n_req, 0);  // tiles per packet if all packets of the request have as many, else -1
        int64_t n_groups_total = 0;
        for (int r = 0; r < n_req; ++r) {
            const kvp_request_t &rq = reqs[r];
            const int n_q = q_offsets[r + 1] - q_offsets[r];
            int64_t pos = 0;
            tile_begin[r] = (int)tiles.size();
            for (int j = 0; j < rq.k; ++j) {
                const int tiles_before = (int)tiles.size();
                auto close_packet = [&]() {
                    const int n = (int)tiles.size() - tiles_before;
                    if (j == 0) pkt_tiles[r] = n;
                    else if (pkt_tiles[r] != n) pkt_tiles[r] = -1;
                };
                auto itp = s->dir.find(rq.packet_ids[j]);
                if (itp == s->dir.end()) return fail(s, KVP_E_NOTFOUND, "request %d: packet %lld not in the store", r, (long long)rq.packet_ids[j]);
                const PacketRec &p = itp->second;
                if (p.compressed()) {
                    // this layer's kept rows, from its own part of the blob (negative stride: V follows
                    // this layer's K); the packet still occupies its span of positions
                    const int rows = p.rows[layer];
                    for (int r0 = 0; r0 < rows; r0 += 64)
                        tiles.push_back(AttnTile{p.layer_off[layer], -rows, r0, std::min(64, rows - r0), (int32_t)pos, 0, 0});
                    pos += p.n_tokens;
                    close_packet();
                    continue;
                }
                // (a packet stored without its header rows: those come from the shared copy, as a tile of their own)
                for (int r0 = 0; r0 < p.head_rows; r0 += 64)
                    tiles.push_back(AttnTile{s->header.elem_off, s->header.stride, r0, std::min(64, p.head_rows - r0), (int32_t)pos, 0, 0});
                for (int r0 = 0; r0 < p.body_rows(); r0 += 64)
                    tiles.push_back(AttnTile{p.elem_off, p.stride, r0, std::min(64, p.body_rows() - r0), (int32_t)pos, 0, 0});
                pos += p.n_tokens;
                close_packet();
            }
            if (pos + n_q > g.max_positions) return fail(s, KVP_E_CAPACITY, "request %d: %lld rows exceed max_positions %d", r, (long long)(pos + n_q), g.max_positions);
            n_pkt_tiles[r] = (int)tiles.size() - tile_begin[r];
            for (int r0 = 0; r0 < n_q; r0 += 64) tiles.push_back(AttnTile{0, 0, r0, std::min(64, n_q - r0), 0, 1, 0});
            metas[r] = ReqMeta{(int32_t)pos, q_offsets[r], n_q, (int32_t)pos};
        }
        // row block, work-item target and launch shape as for the cache path (plan_prefill)
        int bm = MFMA_BM;
        if (s->force_bm == MFMA_BM || s->force_bm == 2 * MFMA_BM) bm = s->force_bm;
        else
            for (int r = 0; r < n_req; ++r)
                if ((int64_t)metas[r].n_q * gq >= 2 * MFMA_BM) bm = 2 * MFMA_BM;
        int64_t n_tiles_total = 0;  // 64-row tiles all the items together will read
        for (int r = 0; r < n_req; ++r) {
            const int64_t blocks = (int64_t)g.n_kv_heads * (((int64_t)metas[r].n_q * gq + bm - 1) / bm);
            n_groups_total += blocks;
            n_tiles_total += blocks * (n_pkt_tiles[r] + (metas[r].n_q + 63) / 64);
        }
        std::vector<AttnGroup> groups;
        std::vector<AttnItem> items;
        int n_slots = 0, part_stride = 1, max_group_rows = 0;
        bool any_split = false, mixed = false;
        const bool split_in_wg = streams_many_tiles(s, n_tiles_total, bm);
        int want = n_groups_total ? (int)std::min<int64_t>(MAX_SPLITS, (target_items(s, n_tiles_total, bm) + n_groups_total - 1) / n_groups_total) : 1;
        if (want < 1) want = 1;
        int per_item0 = 0;  // tiles per item of request 0
        for (int r = 0; r < n_req; ++r) {
            const ReqMeta &rq = metas[r];
            if (rq.n_q == 0) continue;
            const int n_t = n_pkt_tiles[r] + (rq.n_q + 63) / 64;
            int per_item = std::max(4, (n_t + want - 1) / want);  // at least 256 rows per item
            // One request of packets of one length, items shorter than a packet: items that divide a
            // packet evenly never straddle a boundary -- every boundary inside an item re-rotates the
            // query and drains the tile prefetch (16 packets of 8 tiles at 8K: items of 6 tiles 24.3 us
            // per layer, of 4 tiles 23.0).  Items of several packets keep their boundaries whatever
            // their length, and rounding those to whole packets only unbalances them (measured: 8
            // requests of 32 packets, 32 query rows, +4 %).
            if (const int P = pkt_tiles[r]; P > 0 && n_req == 1 && per_item < P) {
                for (int dv = per_item; dv >= 4; --dv)
                    if (P % dv == 0) { per_item = dv; break; }
            }
            if (r == 0) per_item0 = per_item;
            const int M = rq.n_q * gq;
            for (int h = 0; h < g.n_kv_heads; ++h)
                for (int m0 = 0; m0 < M; m0 += bm) {
                    AttnGroup gp;
                    gp.req = r;
                    gp.kv_head = h;
                    gp.m0 = m0;
                    gp.n_rows = std::min(bm, M - m0);
                    const bool half_block = bm == 2 * MFMA_BM && gp.n_rows <= MFMA_BM && s->mixed_blocks;
                    if (half_block) mixed = true;
                    const int t_last = (m0 + gp.n_rows - 1) / gq;
                    const int vis_tiles = n_pkt_tiles[r] + t_last / 64 + 1;  // causal: later query tiles are invisible
                    gp.n_splits = (vis_tiles + per_item - 1) / per_item;
                    gp.part0 = 0;
                    gp.q_off = rq.q_off;
                    gp.pad1 = 0;
                    if (gp.n_splits > 1) {
                        any_split = true;
                        max_group_rows = std::max(max_group_rows, gp.n_rows);
                    }
                    part_stride = std::max(part_stride, gp.n_splits);
                    for (int sp = 0; sp < gp.n_splits; ++sp) {
                        AttnItem it{};
                        it.group = (int)groups.size();
                        it.split = sp;
                        it.kv_begin = tile_begin[r] + sp * per_item;
                        it.kv_end = tile_begin[r] + std::min(vis_tiles, (sp + 1) * per_item);
                        it.half_block = half_block ? 1 : 0;
                        it.req = r;
                        it.kv_head = h;
                        it.m0 = m0;
                        it.n_rows = gp.n_rows;
                        it.ctx_len = rq.ctx_len;
                        it.pos0 = rq.pos0;
                        it.q_off = rq.q_off;
                        it.part_slot = gp.n_splits > 1 ? sp : -1;
                        it.n_q = rq.n_q;
                        items.push_back(it);
                    }
                    groups.push_back(gp);
                }
        }
        assign_part_slots(groups, items, any_split ? part_stride : 0, n_slots);
        const bool shared_rows = xcd_order(items) || n_tiles_total < 16 * (int64_t)s->n_cu;  // (short launches: the hint measured slower)
        AttnInline inl;
        inl.n = 0;
        if (n_req == 1 && metas[0].n_q > 0) {
            fill_inline_items(s, n_req, metas.data(), groups, items, bm, part_stride, per_item0, gq, inl);
        }
        const uint64_t need = (uint64_t)n_slots * (uint64_t)part_slot_bytes(bm, g.head_dim, 1);
        const uint64_t bytes = metas.size() * sizeof(ReqMeta) + groups.size() * sizeof(AttnGroup) +
                               items.size() * sizeof(AttnItem) + tiles.size() * sizeof(AttnTile) + 6 * 64;
        // every check comes before the entry is touched: a call that fails has changed nothing
        if (tot_q > 0 && workspace_bytes < need)
            return fail(s, KVP_E_CAPACITY, "workspace too small: %llu < %llu", (unsigned long long)workspace_bytes, (unsigned long long)need);
        if (!s->dry && tot_q > 0 && need > 0 && (!workspace || ((uintptr_t)workspace & (ALIGN - 1))))
            return fail(s, KVP_E_INVAL, "workspace is null or not 256-byte aligned");
        pk.valid = false;  // the entry's buffer is rewritten below
        pk.last_use = ++s->pf_clock;
        PlanSlot *slot = &pk.own;
        int src = settle_plan_entry(s, pk);
        if (src) return src;
        int hrc = slot->ensure(bytes, s->dry);
        if (hrc) return hip_fail(s, (hipError_t)hrc, "plan buffer");
        PlanWriter w{slot->host, s->dry ? nullptr : slot->dev};
        ReqMeta *rh = w.put<ReqMeta>(metas.size(), &pk.reqs_dev);
        if (!metas.empty()) memcpy(rh, metas.data(), metas.size() * sizeof(ReqMeta));
        AttnGroup *gh = w.put<AttnGroup>(groups.size(), &pk.groups_dev);
        if (!groups.empty()) memcpy(gh, groups.data(), groups.size() * sizeof(AttnGroup));
        AttnItem *ih = w.put<AttnItem>(items.size(), &pk.items_dev);
        if (!items.empty()) memcpy(ih, items.data(), items.size() * sizeof(AttnItem));
        AttnTile *th = w.put<AttnTile>(tiles.size(), &pk.tiles_dev);
        if (!tiles.empty()) memcpy(th, tiles.data(), tiles.size() * sizeof(AttnTile));

        const int n_items_planned = (int)items.size(), n_groups_planned = (int)groups.size();
        {
            kvp_store::DebugPlan &dp = s->dbg_plan;
            const int64_t head[6] = {2, bm, (int64_t)groups.size(), (int64_t)items.size(), n_slots, (int64_t)need};
            memcpy(dp.head, head, sizeof head);
            dp.groups.swap(groups);  // (already copied into the plan buffer above)
            dp.items.swap(items);
            dp.tiles.swap(tiles);
            dp.has_tiles = true;
            dp.inl_n = inl.n;
        }
        pk.slot = slot;
        pk.kind = ATTN_MFMA;
        pk.bm = bm;
        pk.mixed = mixed;
        pk.split_in_wg = split_in_wg;
        pk.shared_rows = shared_rows;
        pk.n_items = n_items_planned;
        pk.n_groups = n_groups_planned;
        pk.tot_q = tot_q;
        pk.any_split = any_split;
        pk.part_stride = part_stride;
        pk.max_group_rows = max_group_rows;
        pk.need = need;
        pk.sig = sig;
        pk.sig_hash = sig_hash;
        pk.stream = hip_stream;
        pk.inl.n = inl.n;
        if (inl.n) pk.inl = inl;
        if (s->dry || tot_q == 0) return KVP_OK;
        int urc = upload_plan(s, slot, w.off, hip_stream);
        if (urc) return urc;
        pk.valid = true;
    } else if (tot_q > 0) {
        if (workspace_bytes < pk.need)
            return fail(s, KVP_E_CAPACITY, "workspace too small: %llu < %llu", (unsigned long long)workspace_bytes, (unsigned long long)pk.need);
        if (pk.need > 0 && (!workspace || ((uintptr_t)workspace & (ALIGN - 1)))) return fail(s, KVP_E_INVAL, "workspace is null or not 256-byte aligned");
    }
    if (s->dry || tot_q == 0) return KVP_OK;

    AttnArgs at;
    memset(&at, 0, sizeof at);
    at.q = q;
    at.k_new = k_new;
    at.v_new = v_new;
    at.cs = s->cs_dev;
    at.prerotated = (flags & KVP_PREROTATED) ? 1 : 0;
    at.tiles = pk.tiles_dev;
    at.arena = s->arena_dev;
    at.k_tail = k_tail;
    at.n_layers_total = g.n_layers;
    at.reqs = pk.reqs_dev;
    at.groups = pk.groups_dev;
    at.items = pk.items_dev;
    at.partials = (float *)workspace;
    at.part_f16 = 1;
    at.out = out;
    at.n_items = pk.n_items;
    at.n_groups = pk.n_groups;
    at.layer = layer;
    at.n_q_heads = g.n_q_heads;
    at.n_kv = g.n_kv_heads;
    at.d = g.head_dim;
    at.bm = pk.bm;
    at.split_in_wg = s->force_split_in_wg >= 0 ? s->force_split_in_wg : (pk.split_in_wg ? 1 : 0);
    at.mixed = pk.mixed ? 1 : 0;
    at.nt_loads = s->nt_loads >= 0 ? s->nt_loads : (pk.shared_rows ? 0 : 1);
    at.part_stride = pk.part_stride;
    at.max_group_rows = pk.max_group_rows;
    at.g = g.n_q_heads / g.n_kv_heads;
    at.scale_log2e = (float)(1.4426950408889634 / sqrt((double)g.head_dim));
    at.inl.n = pk.inl.n;
    if (pk.inl.n) at.inl = pk.inl;
    int e = launch_attention(g.dtype, at, ATTN_MFMA, hip_stream);
    if (e) return hip_fail(s, (hipError_t)e, "attention launch");
    if (pk.any_split) {
        e = launch_combine(g.dtype, at, hip_stream);
        if (e) return hip_fail(s, (hipError_t)e, "combine launch");
    }
    if (in_capture) {
        pk.captured = true;
    } else if (hit) {
        pk.used_since_event = true;
    } else {
        HIP_TRY(s, hipEventRecord(pk.slot->ev, (hipStream_t)hip_stream));
        pk.slot->pending = true;
    }
    return KVP_OK;
}

int kvp_release_captured_plans(kvp_store_t *s)
{
    if (!s) return KVP_E_INVAL;
    int n = 0;
    for (auto *set : {&s->pf_set, &s->pk_set})
        for (auto &e : *set)
            if (e.captured) {
                e.captured = false;
                e.used_since_event = true;  // a replay may still be running: settled before the buffer is rewritten
                ++n;
            }
    return n;
}

int64_t kvp_debug_last_plan(const kvp_store_t *s, int32_t which, int64_t *out, int64_t cap)
{
    if (!s) return KVP_E_INVAL;
    std::vector<int64_t> tiles;
    if (which == 0) {
        // the gather's tiles, as the kernel derives them from the segment list:
        // src_base, stride, first row in the segment, rows, cache row, Delta, request, layer (layered lists)
        tiles.push_back(0);
        for (const AsmSeg &g : s->dbg_segs)
            for (int t0 = 0; t0 < g.n_rows; t0 += s->dbg_tile_rows) {
                int64_t row[8] = {g.src_base, g.stride, t0, std::min(s->dbg_tile_rows, g.n_rows - t0), g.dst_row + t0,
                                  g.pos, g.req, s->dbg_layered ? g.layer : -1};
                tiles.insert(tiles.end(), row, row + 8);
                ++tiles[0];
            }
    }
    if (which == 2) {  // how many of the last prefill plan's items ride in the kernel arguments
        tiles.push_back(s->dbg_plan.inl_n);
    } else if (which != 0) {
        // the last prefill plan: head, then groups (6 numbers each), items (4 each) and, for the
        // in-place path, the tile count and the tiles (6 each)
        const kvp_store::DebugPlan &dp = s->dbg_plan;
        tiles.assign(dp.head, dp.head + 6);
        for (const AttnGroup &x : dp.groups) {
            int64_t row[6] = {x.req, x.kv_head, x.m0, x.n_rows, x.part0, x.n_splits};
            tiles.insert(tiles.end(), row, row + 6);
        }
        for (const AttnItem &x : dp.items) {
            int64_t row[4] = {x.group, x.split, x.kv_begin, x.kv_end};
            tiles.insert(tiles.end(), row, row + 4);
        }
        if (dp.has_tiles) {
            tiles.push_back((int64_t)dp.tiles.size());
            for (const AttnTile &x : dp.tiles) {
                int64_t row[6] = {x.src_base, x.stride, x.row0, x.n_rows, x.pos, x.kind};
                tiles.insert(tiles.end(), row, row + 6);
            }
        }
    }
    const std::vector<int64_t> &v = tiles;
    for (int64_t i = 0; i < (int64_t)v.size() && i < cap && out; ++i) out[i] = v[i];
    return (int64_t)v.size();
}

}  // extern "C"
