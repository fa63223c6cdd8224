/*
 * kvp_oracle.c -- CPU oracle for the KV Packet serving hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the serving path computes.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product library never does,
 * and the two share no code.
 *
 * What it follows (KV Packet paper):
 *   - Sec. 4.1, Eq. 2: a packet is the KV of [header, document, trailer]
 *     tokens, computed once and frozen.
 *   - Sec. 3.1, Eq. 1: a key cached at position S is moved to S+Delta by one
 *     RoPE rotation R_{Theta,Delta}; values are not position-encoded.
 *   - Sec. 4.2.1, step 4: the packets' caches are realigned with Eq. 1 and
 *     concatenated into one cache; the query tokens then run with causal
 *     attention and see every earlier token.
 *
 * Readings where the paper is silent (all restated in the design notes):
 *   - a packet's keys are cached at local positions 0..len-1, so the rotation
 *     offset of the j-th retrieved packet is its destination start row;
 *   - adapter rows occupy positions like any other row (Fig. 5 caption);
 *   - RoPE pairs element i with element i + d/2, theta_i = base^(-2i/d);
 *   - rotation arithmetic is fp32 with each product and each sum rounded
 *     separately (no fused multiply-add), cos/sin are double-precision libm
 *     values of (double)pos * (double)inv_freq[i] rounded to fp32, and the
 *     result is rounded to nearest-even into the cache dtype;
 *   - softmax scale 1/sqrt(d); query head hq reads KV head hq / g.
 *
 * Attention accumulates in fp64 over the oracle's own rounded cache.
 *
 * Parity status: every function here is pinned by tests/test_oracle_pins.py
 * (brute force with explicit rotation matrices, rotation composition,
 * relative-position property, reduction to plain causal attention checked
 * against a library SDPA, concatenation-by-hand, order permutation, softmax
 * invariants, closed-form flop count).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KVO_F32 0
#define KVO_BF16 1

static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* round-to-nearest-even fp32 -> bf16; inputs are finite by contract */
static uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

static size_t elem_size(int dtype) { return dtype == KVO_BF16 ? 2 : 4; }

static float load_elem(const void *p, int dtype, size_t i)
{
    if (dtype == KVO_BF16)
        return bf16_bits_to_f32(((const uint16_t *)p)[i]);
    return ((const float *)p)[i];
}

static void store_elem(void *p, int dtype, size_t i, float x)
{
    if (dtype == KVO_BF16)
        ((uint16_t *)p)[i] = f32_to_bf16_bits(x);
    else
        ((float *)p)[i] = x;
}

/* theta_i = base^(-2i/d), i in [0, d/2): computed in double, kept as fp32. */
void kvo_inv_freq(double rope_base, int d, float *inv_freq)
{
    for (int i = 0; i < d / 2; ++i)
        inv_freq[i] = (float)pow(rope_base, -2.0 * (double)i / (double)d);
}

/* cos and sin of pos * theta_i (Eq. 1's rotation angle for offset pos). */
void kvo_cos_sin(int64_t pos, const float *inv_freq, int d, float *c, float *s)
{
    for (int i = 0; i < d / 2; ++i) {
        double a = (double)pos * (double)inv_freq[i];
        c[i] = (float)cos(a);
        s[i] = (float)sin(a);
    }
}

/* y = R x for one head vector: 2x2 rotation of each (x[i], x[i+d/2]) pair.
 * volatile temporaries keep every product and sum separately rounded. */
void kvo_rotate(const float *x, int d, const float *c, const float *s, float *y)
{
    int h = d / 2;
    for (int i = 0; i < h; ++i) {
        volatile float xc = x[i] * c[i];
        volatile float ys = x[i + h] * s[i];
        volatile float yc = x[i + h] * c[i];
        volatile float xs = x[i] * s[i];
        float lo = xc - ys;
        float hi = yc + xs;
        y[i] = lo;
        y[i + h] = hi;
    }
}

/*
 * Realign and concatenate k packets for ONE request (Sec. 4.2.1 step 4).
 *   pk_k[j], pk_v[j] : packet j's K and V, [n_layers][n_kv][lens[j]][d], dtype
 *   k_out, v_out     : [n_layers][n_kv][t_cap][d], dtype; rows
 *                      base_pos .. base_pos+T-1 are written, others untouched
 * Returns base_pos + T (the context length), or -1 if it exceeds t_cap.
 */
int64_t kvo_assemble(int dtype, int n_layers, int n_kv, int d,
                     const float *inv_freq, int k,
                     const void *const *pk_k, const void *const *pk_v,
                     const int32_t *lens, int64_t base_pos, int64_t t_cap,
                     void *k_out, void *v_out)
{
    int64_t end = base_pos;
    for (int j = 0; j < k; ++j)
        end += lens[j];
    if (end > t_cap || base_pos < 0)
        return -1;

    size_t es = elem_size(dtype);
    int64_t delta = base_pos; /* Delta_j: destination start row of packet j */
    for (int j = 0; j < k; ++j) {
        int len = lens[j];
        float *c = (float *)malloc(sizeof(float) * (size_t)(d / 2 + 1));
        float *s = (float *)malloc(sizeof(float) * (size_t)(d / 2 + 1));
        kvo_cos_sin(delta, inv_freq, d, c, s);
#pragma omp parallel for collapse(2) schedule(static)
        for (int l = 0; l < n_layers; ++l) {
            for (int h = 0; h < n_kv; ++h) {
                float x[1024], y[1024];
                size_t src0 = ((size_t)l * n_kv + h) * (size_t)len * d;
                size_t dst0 = (((size_t)l * n_kv + h) * (size_t)t_cap + (size_t)delta) * d;
                for (int t = 0; t < len; ++t) {
                    for (int e = 0; e < d; ++e)
                        x[e] = load_elem(pk_k[j], dtype, src0 + (size_t)t * d + e);
                    kvo_rotate(x, d, c, s, y);
                    for (int e = 0; e < d; ++e)
                        store_elem(k_out, dtype, dst0 + (size_t)t * d + e, y[e]);
                }
                /* values carry no position: bit copy */
                memcpy((char *)v_out + dst0 * es,
                       (const char *)pk_v[j] + src0 * es, (size_t)len * d * es);
            }
        }
        free(c);
        free(s);
        delta += len;
    }
    return end;
}

/*
 * Query side of one layer: rotate Q and K_new from position 0 to ctx_len + t
 * (skipped when prerotated != 0), append K_new (rounded to dtype) and V_new
 * at cache rows ctx_len + t.
 *   q      : [n_q][n_q_heads][d] dtype      k_new, v_new : [n_q][n_kv][d] dtype
 *   k_layer, v_layer : [n_kv][t_cap][d] dtype
 *   q_rot  : out, [n_q][n_q_heads][d] fp32 (the rotated query is kept in fp32)
 */
void kvo_query_rope_append(int dtype, int n_q_heads, int n_kv, int d,
                           const float *inv_freq, int n_q, int64_t ctx_len,
                           const void *q, const void *k_new, const void *v_new,
                           int prerotated, void *k_layer, void *v_layer,
                           int64_t t_cap, float *q_rot)
{
    size_t es = elem_size(dtype);
    float c[512], s[512], x[1024], y[1024];
    for (int t = 0; t < n_q; ++t) {
        int64_t pos = ctx_len + t;
        kvo_cos_sin(pos, inv_freq, d, c, s);
        for (int hq = 0; hq < n_q_heads; ++hq) {
            size_t o = ((size_t)t * n_q_heads + hq) * d;
            for (int e = 0; e < d; ++e)
                x[e] = load_elem(q, dtype, o + e);
            if (prerotated)
                memcpy(y, x, sizeof(float) * (size_t)d);
            else
                kvo_rotate(x, d, c, s, y);
            memcpy(q_rot + o, y, sizeof(float) * (size_t)d);
        }
        for (int h = 0; h < n_kv; ++h) {
            size_t o = ((size_t)t * n_kv + h) * d;
            size_t dst = ((size_t)h * (size_t)t_cap + (size_t)pos) * d;
            for (int e = 0; e < d; ++e)
                x[e] = load_elem(k_new, dtype, o + e);
            if (prerotated)
                memcpy(y, x, sizeof(float) * (size_t)d);
            else
                kvo_rotate(x, d, c, s, y);
            for (int e = 0; e < d; ++e)
                store_elem(k_layer, dtype, dst + e, y[e]);
            memcpy((char *)v_layer + dst * es, (const char *)v_new + o * es, (size_t)d * es);
        }
    }
}

/*
 * Compressed packets (Sec. 5.4: pruning keeps a different subset of a packet's rows in every
 * layer, and the packet stays an opaque unit).  One layer of the composed cache: packet j kept
 * rows[j] of its rows in this layer and still occupies spans[j] positions, so its keys are
 * rotated by Delta_j = base_pos + sum of the spans before it (Eq. 1 needs no position of the
 * single row: a kept key carries the rotation of the local position it was cached at), while
 * its rows land right behind the kept rows of the packets before it.
 *   pk_k[j], pk_v[j] : [n_kv][rows[j]][d] dtype      k_out, v_out : [n_kv][t_cap][d] dtype
 * Returns the number of rows written (or -1 if they exceed t_cap); *pos_end = base_pos + sum of
 * the spans, the position of the first token after the packets.
 */
int64_t kvo_assemble_layer_spans(int dtype, int n_kv, int d, const float *inv_freq, int k,
                                 const void *const *pk_k, const void *const *pk_v,
                                 const int32_t *rows, const int32_t *spans, int64_t base_pos,
                                 int64_t t_cap, void *k_out, void *v_out, int64_t *pos_end)
{
    int64_t total = 0;
    for (int j = 0; j < k; ++j)
        total += rows[j];
    if (total > t_cap || base_pos < 0)
        return -1;
    size_t es = elem_size(dtype);
    float c[512], s[512], x[1024], y[1024];
    int64_t row0 = 0;         /* destination row of packet j's first kept row */
    int64_t delta = base_pos; /* Delta_j */
    for (int j = 0; j < k; ++j) {
        kvo_cos_sin(delta, inv_freq, d, c, s);
        for (int h = 0; h < n_kv; ++h) {
            size_t src0 = (size_t)h * (size_t)rows[j] * d;
            size_t dst0 = ((size_t)h * (size_t)t_cap + (size_t)row0) * d;
            for (int t = 0; t < rows[j]; ++t) {
                for (int e = 0; e < d; ++e)
                    x[e] = load_elem(pk_k[j], dtype, src0 + (size_t)t * d + e);
                kvo_rotate(x, d, c, s, y);
                for (int e = 0; e < d; ++e)
                    store_elem(k_out, dtype, dst0 + (size_t)t * d + e, y[e]);
            }
            memcpy((char *)v_out + dst0 * es, (const char *)pk_v[j] + src0 * es,
                   (size_t)rows[j] * d * es);
        }
        row0 += rows[j];
        delta += spans[j];
    }
    *pos_end = delta;
    return total;
}

/*
 * Query side of one layer when rows and positions differ (compressed packets): query token t
 * sits at position pos0 + t and its K_new / V_new are appended at cache row row0 + t.
 * Arguments otherwise as kvo_query_rope_append.
 */
void kvo_query_rope_append_at(int dtype, int n_q_heads, int n_kv, int d,
                              const float *inv_freq, int n_q, int64_t row0, int64_t pos0,
                              const void *q, const void *k_new, const void *v_new,
                              int prerotated, void *k_layer, void *v_layer,
                              int64_t t_cap, float *q_rot)
{
    size_t es = elem_size(dtype);
    float c[512], s[512], x[1024], y[1024];
    for (int t = 0; t < n_q; ++t) {
        kvo_cos_sin(pos0 + t, inv_freq, d, c, s);
        for (int hq = 0; hq < n_q_heads; ++hq) {
            size_t o = ((size_t)t * n_q_heads + hq) * d;
            for (int e = 0; e < d; ++e)
                x[e] = load_elem(q, dtype, o + e);
            if (prerotated)
                memcpy(y, x, sizeof(float) * (size_t)d);
            else
                kvo_rotate(x, d, c, s, y);
            memcpy(q_rot + o, y, sizeof(float) * (size_t)d);
        }
        for (int h = 0; h < n_kv; ++h) {
            size_t o = ((size_t)t * n_kv + h) * d;
            size_t dst = ((size_t)h * (size_t)t_cap + (size_t)(row0 + t)) * d;
            for (int e = 0; e < d; ++e)
                x[e] = load_elem(k_new, dtype, o + e);
            if (prerotated)
                memcpy(y, x, sizeof(float) * (size_t)d);
            else
                kvo_rotate(x, d, c, s, y);
            for (int e = 0; e < d; ++e)
                store_elem(k_layer, dtype, dst + e, y[e]);
            memcpy((char *)v_layer + dst * es, (const char *)v_new + o * es, (size_t)d * es);
        }
    }
}

/*
 * Softmax attention of the n_q query tokens over one layer's cache, by the
 * definition: query token t (at row ctx_len + t) sees rows 0 .. ctx_len + t.
 *   q_rot : [n_q][n_q_heads][d] fp32       out : [n_q][n_q_heads][d] fp64
 */
void kvo_attention(int dtype, int n_q_heads, int n_kv, int d, int n_q,
                   int64_t ctx_len, const float *q_rot, const void *k_layer,
                   const void *v_layer, int64_t t_cap, double *out)
{
    int g = n_q_heads / n_kv;
    double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int t = 0; t < n_q; ++t) {
        for (int hq = 0; hq < n_q_heads; ++hq) {
            int h = hq / g;
            int64_t n_vis = ctx_len + t + 1;
            const float *qv = q_rot + ((size_t)t * n_q_heads + hq) * d;
            double *score = (double *)malloc(sizeof(double) * (size_t)n_vis);
            double m = -INFINITY;
            for (int64_t u = 0; u < n_vis; ++u) {
                size_t row = ((size_t)h * (size_t)t_cap + (size_t)u) * d;
                double acc = 0.0;
                for (int e = 0; e < d; ++e)
                    acc += (double)qv[e] * (double)load_elem(k_layer, dtype, row + e);
                score[u] = acc * scale;
                if (score[u] > m)
                    m = score[u];
            }
            double denom = 0.0;
            double *o = out + ((size_t)t * n_q_heads + hq) * d;
            for (int e = 0; e < d; ++e)
                o[e] = 0.0;
            for (int64_t u = 0; u < n_vis; ++u) {
                double p = exp(score[u] - m);
                denom += p;
                size_t row = ((size_t)h * (size_t)t_cap + (size_t)u) * d;
                for (int e = 0; e < d; ++e)
                    o[e] += p * (double)load_elem(v_layer, dtype, row + e);
            }
            for (int e = 0; e < d; ++e)
                o[e] /= denom;
            free(score);
        }
    }
}

/* Number of OpenMP threads the parallel loops above will use. */
#ifdef _OPENMP
#include <omp.h>
int kvo_num_threads(void) { return omp_get_max_threads(); }
#else
int kvo_num_threads(void) { return 1; }
#endif
