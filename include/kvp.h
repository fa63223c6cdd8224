/*
 * kvp.h -- C ABI of the KV Packet serving hot path on MI355X (gfx950).
 *
 * The library composes independently precomputed document KV "packets" into
 * one context cache and runs the query tokens' attention over it:
 *
 *     kvp_store_put      keep a packet (Sec. 4.1, Eq. 2) in an HBM-resident store
 *     kvp_assemble       realign the retrieved packets' keys with one RoPE rotation
 *                        each (Sec. 3.1, Eq. 1) and concatenate K and V into a
 *                        per-layer cache, with no recomputation (Sec. 4.1; Sec. 4.2.1
 *                        step 4)
 *     kvp_query_prefill  causal attention of the query tokens over that cache: full
 *                        over the packet prefix, causal among themselves (Sec. 4.2.1
 *                        step 4; Fig. 2(d))
 *     kvp_prefill_packets   the same attention read in place from the store, no cache
 *     kvp_store_put_compressed, kvp_store_put_header / _body   packets pruned per layer
 *                        (Sec. 5.4); the global header's rows stored once (Sec. 4.1)
 *
 * Conventions
 *   - Every pointer is labelled HOST or DEVICE.  The caller owns every DEVICE buffer
 *     (arena, caches, Q/K/V, outputs, workspace); the library owns only host metadata
 *     and small device tables it allocates itself (cos/sin table, per-call plans).
 *   - `hip_stream` is a raw hipStream_t (NULL = the default stream).  Calls are
 *     asynchronous on it; only validation errors are synchronous.  All validation
 *     happens on the host before anything is launched: a call that fails has changed
 *     nothing.
 *   - Stream capture: kvp_query_prefill and kvp_prefill_packets may be captured into a HIP
 *     graph once a call with the same geometry (context lengths, query offsets, block table;
 *     for kvp_prefill_packets the same requests) has run on the same stream outside capture:
 *     that call built and uploaded the plan, the captured call only launches from it, and the
 *     store keeps that plan unchanged until it is destroyed.  kvp_assemble may be captured when
 *     its plan rides in the kernel arguments: a contiguous cache and at most 80 segments over
 *     all requests (a whole packet is one segment, a header-less packet two, a compressed
 *     packet one per layer).  A call that cannot be
 *     captured returns KVP_E_INVAL and launches nothing.  Host-side results (ctx_len, ctx_rows)
 *     are written when the call is captured, not when the graph runs.
 *   - A stream handed to kvp_query_prefill or kvp_prefill_packets must stay alive until the store
 *     is destroyed: the store puts an event behind that stream's work before it rewrites a plan
 *     the stream's launches read.
 *   - A store is thread-compatible: one thread at a time per store.
 *   - Return value: 0 (KVP_OK) or a negative kvp_status; text via kvp_last_error().
 *   - Tensors are dense row-major in the order written, innermost index last.
 *   - dtype KVP_BF16: elements are bfloat16 bit patterns; arithmetic is fp32.
 *
 * Positions (Sec. 4.2.1 step 4 with Eq. 1; Fig. 5 caption: adapter rows occupy
 * positions).  A packet's keys are stored rotated at its local positions
 * 0..n_tokens-1, header row first.  The j-th retrieved packet of a request lands at
 * rows Delta_j = base_pos + sum_{i<j} n_tokens_i, and its keys are rotated by
 * R_{Theta,Delta_j}.  A cache row index IS the absolute position.  Query token t of a
 * request sits at position ctx_len + t.
 *
 * RoPE convention: element i pairs with element i + head_dim/2; theta_i =
 * rope_base^(-2i/head_dim) rounded to fp32 (or the caller's inv_freq).  cos/sin are
 * double-precision libm values of (double)pos * (double)theta_i rounded to fp32; the
 * rotation is fp32 with every product and sum rounded separately; results are rounded
 * to nearest-even into the cache dtype.  Values are never rotated.
 */
#ifndef KVP_H
#define KVP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvp_store kvp_store_t; /* opaque */

enum kvp_dtype { KVP_F32 = 0, KVP_BF16 = 1 };
enum kvp_layout { KVP_CONTIG = 0, KVP_PAGED = 1 };

enum kvp_status {
    KVP_OK = 0,
    KVP_E_INVAL = -1,    /* null pointer, bad shape, odd head_dim, unknown dtype/layout */
    KVP_E_EXISTS = -2,   /* packet id already stored (packets are immutable) */
    KVP_E_NOTFOUND = -3, /* unknown packet id */
    KVP_E_NOSPACE = -4,  /* arena full */
    KVP_E_CAPACITY = -5, /* context does not fit t_cap / block table / max_positions /
                            workspace */
    KVP_E_HIP = -6       /* HIP runtime failure */
};

/* flags of kvp_query_prefill */
#define KVP_PREROTATED 1u /* q and k_new already carry RoPE at ctx_len + t */

/* device = KVP_DEVICE_NONE builds a store that validates and plans but owns no GPU
 * state and launches nothing (host-logic tests on machines without a GPU). */
#define KVP_DEVICE_NONE (-1)

typedef struct {
    int32_t n_layers, n_q_heads, n_kv_heads, head_dim; /* head_dim even, <= 256;
                                                          n_q_heads % n_kv_heads == 0 */
    int32_t n_header, n_trailer; /* N_h, N_t of Eq. 2.  Adapter rows are ordinary rows at serving
                                    time; n_header is used only by kvp_store_put_header /
                                    kvp_store_put_body (header rows stored once) */
    int32_t dtype;               /* kvp_dtype of store, caches, Q, K_new, V_new, O */
    int32_t max_positions;       /* bound on ctx_len + n_q; sizes the cos/sin table */
    double rope_base;
    const float *inv_freq; /* HOST, nullable, [head_dim/2]; replaces rope_base */
    void *arena;           /* caller-owned packet storage, 256-byte aligned: DEVICE memory, or pinned
                            * HOST memory mapped into the device (hipHostMalloc, torch pin_memory):
                            * the tier the paper keeps its packets in (Sec. 5.1); the kernels then
                            * read the packets over PCIe, in place, at every assembly */
    uint64_t arena_bytes;
    int32_t device; /* HIP device ordinal, or KVP_DEVICE_NONE */
} kvp_config_t;

/* Creates a store over the caller's arena.  Builds the [max_positions][head_dim/2]
 * cos/sin table on the host and uploads it.  *out is untouched on failure (the error
 * text is then available through kvp_last_error(NULL)). */
int kvp_store_create(const kvp_config_t *cfg, kvp_store_t **out);

/* Frees host state and the library's own device tables; never the arena.  Waits for
 * the work it has launched. */
int kvp_store_destroy(kvp_store_t *store);

/*
 * Sec. 4.1, Eq. 2: stores one packet, the K and V of [header, document, trailer] rows.
 *   k, v : [n_layers][n_kv_heads][n_tokens][head_dim], HOST (src_on_device == 0) or
 *          DEVICE (!= 0); K already rotated at local positions 0..n_tokens-1.
 * The data is copied into the arena (asynchronously for DEVICE sources; the caller
 * keeps k, v alive until the stream has passed the copy).  In the arena a packet is one
 * 256-byte aligned blob: K [n_layers][n_kv_heads][n_tokens][head_dim] then V likewise,
 * so each (layer, head) of a packet is one contiguous run for the gather.
 * Errors: KVP_E_INVAL (null, n_tokens < 1, id < 0), KVP_E_EXISTS, KVP_E_NOSPACE.
 */
int kvp_store_put(kvp_store_t *store, int64_t packet_id, int32_t n_tokens, const void *k,
                  const void *v, int32_t src_on_device, void *hip_stream);

/*
 * Sec. 5.4 (compatibility with KV compression): a packet whose rows were pruned, with a
 * different subset kept in every layer, stays an opaque unit that is realigned and
 * concatenated like any other.  n_rows[l] (HOST, [n_layers], each in [0, span]) rows survive in
 * layer l; the packet still occupies `span` positions (its uncompressed length), so the
 * packets after it and the query keep the positions they would have without compression, and
 * Eq. 1 rotates every kept key by the packet's Delta_j (a kept key carries the rotation of the
 * local position it was cached at; no per-row position is needed).  In the composed cache the
 * kept rows of a layer follow each other without gaps, so layers have different row counts
 * (kvp_cache_t.ctx_rows).
 * k, v: layer after layer, layer l as [n_kv_heads][n_rows[l]][head_dim].
 * Other arguments, copies and errors as kvp_store_put.  kvp_prefill_packets reads, for the
 * layer it is called for, the rows that layer kept.
 */
int kvp_store_put_compressed(kvp_store_t *store, int64_t packet_id, int32_t span, const int32_t *n_rows,
                             const void *k, const void *v, int32_t src_on_device, void *hip_stream);

/*
 * Sec. 4.1: the adapters are global, shared by all documents, and the header comes first in
 * Eq. 2; under causal attention its K and V at local positions 0..n_header-1 are therefore the
 * same in every packet.  A store may hold them once:
 *   kvp_store_put_header : k, v [n_layers][n_kv_heads][n_header][head_dim] (n_header of the
 *                          config, >= 1), K rotated at local positions 0..n_header-1; once per
 *                          store (KVP_E_EXISTS after that).
 *   kvp_store_put_body   : a packet without its header rows.  n_tokens is its full length, header
 *                          included (the positions it occupies); k, v hold its rows n_header ..
 *                          n_tokens-1 as [n_layers][n_kv_heads][n_tokens - n_header][head_dim],
 *                          K rotated at those local positions.  Needs the header to be stored and
 *                          n_tokens > n_header (KVP_E_INVAL otherwise).
 * kvp_assemble and kvp_prefill_packets read the header rows of such a packet from the shared
 * copy and rotate them by the packet's own Delta_j; results are those of the whole packet
 * stored with kvp_store_put.  Whole and header-less packets may be mixed in a store and in a
 * request.  Other arguments, copies and errors as kvp_store_put.
 */
int kvp_store_put_header(kvp_store_t *store, const void *k, const void *v, int32_t src_on_device,
                         void *hip_stream);
int kvp_store_put_body(kvp_store_t *store, int64_t packet_id, int32_t n_tokens, const void *k,
                       const void *v, int32_t src_on_device, void *hip_stream);

/* Rows of a stored packet (for a compressed packet: the positions it occupies), or
 * KVP_E_NOTFOUND. */
int32_t kvp_store_packet_len(const kvp_store_t *store, int64_t packet_id);
/* Rows a stored packet holds in one layer (its length, unless compressed), or KVP_E_NOTFOUND /
 * KVP_E_INVAL. */
int32_t kvp_store_packet_rows(const kvp_store_t *store, int64_t packet_id, int32_t layer);
/* Bytes of the arena in use. */
uint64_t kvp_store_bytes_used(const kvp_store_t *store);
/* 1 if the arena is pinned host memory (packets are read over PCIe), 0 if device memory. */
int32_t kvp_store_arena_on_host(const kvp_store_t *store);
/* Arena bytes a packet of n_tokens rows takes (alignment included). */
uint64_t kvp_packet_bytes(const kvp_config_t *cfg, int32_t n_tokens);

typedef struct {
    const int64_t *packet_ids; /* HOST [k], concatenation order; repeats allowed */
    int32_t k;                 /* 0 allowed: no documents */
    int32_t base_pos;          /* position of the first packet row (>= 0); rows below it
                                  belong to the caller (e.g. a prompt prefix) */
} kvp_request_t;

typedef struct {
    int32_t layout; /* kvp_layout */
    /* DEVICE.  CONTIG: [n_req][n_layers][n_kv_heads][t_cap][head_dim]
     *          PAGED : pool [n_layers][n_blocks][n_kv_heads][block_size][head_dim];
     *                  logical row p of request r lives in block
     *                  block_table[r][p / block_size], slot p % block_size        */
    void *k, *v;
    int32_t t_cap;                 /* CONTIG */
    int32_t n_blocks, block_size;  /* PAGED; block_size a power of two */
    const int32_t *block_table;    /* PAGED: HOST [n_req][max_blocks_per_req] */
    int32_t max_blocks_per_req;
    int32_t *ctx_len; /* HOST [n_req].  Written by kvp_assemble (base_pos + T); read by
                         kvp_query_prefill, which does not change it: after the last
                         layer the caller adds n_q. */
    int32_t *ctx_rows; /* HOST [n_req][n_layers], or NULL.  Rows of the composed cache per layer.
                          They differ from ctx_len (a position) only when a request names a
                          compressed packet (kvp_store_put_compressed); such requests need this
                          array.  Written by kvp_assemble for the layers it assembles, read by
                          kvp_query_prefill; after the last layer the caller adds n_q to every
                          entry as well. */
} kvp_cache_t;

/*
 * Sec. 3.1, Eq. 1 and Sec. 4.2.1 step 4: for every request r, packet j, layer l in
 * [layer_begin, layer_end), KV head h, row t:
 *     K_cache[r][l][h][Delta_j + t] = round(R_{Theta,Delta_j} K_packet[l][h][t])
 *     V_cache[r][l][h][Delta_j + t] = V_packet[l][h][t]            (bit copy)
 * All requested layers go in ONE launch.  Rows outside [base_pos, base_pos + T) are not
 * touched.  cache->ctx_len[r] = base_pos + T on success.
 * Errors: KVP_E_INVAL, KVP_E_NOTFOUND, KVP_E_CAPACITY.
 */
int kvp_assemble(kvp_store_t *store, const kvp_request_t *reqs, int32_t n_req,
                 int32_t layer_begin, int32_t layer_end, kvp_cache_t *cache,
                 void *hip_stream);

/*
 * Sec. 4.2.1 step 4 (Fig. 2(d)): one layer of the query forward's attention.
 *   q            : DEVICE [tot_q][n_q_heads][head_dim]
 *   k_new, v_new : DEVICE [tot_q][n_kv_heads][head_dim]
 *   q_offsets    : HOST [n_req + 1]; request r owns query rows q_offsets[r] ..
 *                  q_offsets[r+1]-1 (n_q may be 0)
 *   out          : DEVICE [tot_q][n_q_heads][head_dim]
 * Unless KVP_PREROTATED, q and k_new are rotated from position 0 to ctx_len[r] + t.
 * K_new (rounded to the cache dtype) and V_new are appended at cache rows ctx_len[r] + t,
 * then for query head hq (KV head hq / (n_q_heads / n_kv_heads)):
 *     out[t][hq] = softmax_{u <= ctx_len + t}(q_t . K[u] / sqrt(head_dim)) V[u]
 * workspace: DEVICE scratch of at least kvp_prefill_workspace_bytes(); contents are
 * undefined afterwards.
 * Errors: KVP_E_INVAL, KVP_E_CAPACITY (cache, block table, max_positions or workspace
 * too small).
 */
int kvp_query_prefill(kvp_store_t *store, kvp_cache_t *cache, int32_t layer, const void *q,
                      const void *k_new, const void *v_new, const int32_t *q_offsets,
                      int32_t n_req, uint32_t flags, void *workspace,
                      uint64_t workspace_bytes, void *out, void *hip_stream);

/*
 * The same attention without materialising a cache (Sec. 3.1: the score of two tokens
 * depends only on their position difference, so instead of rotating every cached key by
 * Delta_j (Eq. 1) the query is rotated by (ctx_len + t) - Delta_j for packet j's rows).
 * K and V are read in place from the store; nothing is gathered or written except
 *   k_tail : DEVICE [tot_q][n_kv_heads][head_dim], out: K_new rotated to ctx_len[r] + t and
 *            rounded exactly as kvp_query_prefill would have appended it (V_new needs no
 *            copy); the caller keeps it if decoding continues.
 * `out` equals what kvp_assemble + kvp_query_prefill give, within the attention tolerance
 * (operands are rounded to bf16 at different points).  reqs[r].base_pos must be 0: rows below
 * base_pos are rows the caller wrote into a cache, and this path has none to read them from; a
 * prompt that precedes the documents is stored as a packet of its own and named first (it lands
 * at Delta = 0, which rotates nothing: the same composition).  bf16 stores with head_dim 128
 * only.  workspace as for kvp_query_prefill.
 * Errors: KVP_E_INVAL, KVP_E_NOTFOUND, KVP_E_CAPACITY.
 */
int kvp_prefill_packets(kvp_store_t *store, const kvp_request_t *reqs, int32_t n_req, int32_t layer,
                        const void *q, const void *k_new, const void *v_new, const int32_t *q_offsets,
                        uint32_t flags, void *k_tail, void *workspace, uint64_t workspace_bytes,
                        void *out, void *hip_stream);

/*
 * kvp_query_prefill for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same computation with the same kernels, but the
 * split-KV partial results, the generic kernel's rotated query and the call's plan live in a static
 * device array of the library instead of a caller workspace and a library-allocated plan buffer:
 * the call makes no hipMalloc / hipFree (nor any other allocating call), on a plan it has seen
 * before or on a new one.  The array (32 MiB per GPU, held by every GPU the library has a store on
 * until the process ends) gives kvp_static_workspace_bytes() = 31 MiB of workspace and 1 MiB for the
 * plan; a call that needs more of either returns KVP_E_CAPACITY and launches nothing (the
 * metric's 8K-context request needs 5.7 MiB, eight 16.9K-context requests of 128 query rows
 * together 16.5 MiB; the split counts the planner chooses by itself keep a call's partial rows
 * under about 26 MiB, so only calls cut finer through a tuning knob exceed the array).  Arguments,
 * results and other errors as kvp_query_prefill, without `workspace`.
 * All calls on one GPU share that GPU's array, whichever store or stream they come from, and the
 * array keeps the last call's contents: calls are correct one after the other in stream order
 * (each call first replaces the plan if it differs from the one the array holds, and every
 * partial result is written before it is read; nothing needs clearing), and calls that overlap
 * on one GPU -- on two streams, or a captured graph replayed after another call has replaced its
 * plan -- race.  kvp_query_prefill is unaffected by it and may overlap freely.
 */
int kvp_query_prefill_static(kvp_store_t *store, kvp_cache_t *cache, int32_t layer, const void *q,
                             const void *k_new, const void *v_new, const int32_t *q_offsets, int32_t n_req,
                             uint32_t flags, void *out, void *hip_stream);
/* Workspace bytes the static array offers a kvp_query_prefill_static call (compare with
 * kvp_prefill_workspace_bytes). */
uint64_t kvp_static_workspace_bytes(void);

/* Stream capture keeps the plan a captured kvp_query_prefill / kvp_prefill_packets launches from
 * (at most 64 per entry point and store; a capture beyond that returns KVP_E_CAPACITY).  Once the
 * graphs that were captured on this store have been destroyed, this call makes those plans
 * replaceable again.  Returns the number of plans released, or KVP_E_INVAL. */
int kvp_release_captured_plans(kvp_store_t *store);

/* Upper bound of the workspace kvp_query_prefill needs for n_req requests with at most
 * max_tot_q query rows in total and contexts (ctx_len + n_q) of at most max_ctx rows. */
uint64_t kvp_prefill_workspace_bytes(const kvp_store_t *store, int32_t n_req,
                                     int32_t max_tot_q, int32_t max_ctx);

/* Text of the last error on this store (store == NULL: of the last failed
 * kvp_store_create on this thread).  Valid until the next call on the store. */
const char *kvp_last_error(const kvp_store_t *store);

/* Host-logic introspection (tests): copies up to cap int64 words describing the plan of
 * the last kvp_assemble (which == 0) or kvp_query_prefill / kvp_prefill_packets (which == 1) and
 * returns the number of words the full description has.  Layout: see kvp_plan.h in the sources.
 * which == 2: one word, the number of work items of that prefill plan that the workgroups
 * rebuild from their index (regular launches for one request), 0 if they read them from memory. */
int64_t kvp_debug_last_plan(const kvp_store_t *store, int32_t which, int64_t *out,
                            int64_t cap);

/* Library version, e.g. "kvp 0.1 gfx950". */
const char *kvp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVP_H */
