/*
 * prism_oracle.c — CPU oracle (TEST INFRASTRUCTURE ONLY; see prism_oracle.h).
 *
 * Plain C, fp64 arithmetic, no blocking, no fusion, no reordering: each function
 * is the definition written out so it can be checked against the paper by eye.
 *
 *   Pool / balloon bookkeeping  — paper Sec. 4.2: D1 (per-model limits grow and
 *       shrink, memory only changes hands), D2 (token blocks go to slots inside
 *       pages; models never share a page), D3 (2 MB pages, partially filled
 *       pages first).  The paper fixes no tie-breaks; the ones used here are
 *       LIFO free stack, newest-empty-frame-first reclaim, lowest-slot-first
 *       placement.
 *   Decode attention            — paper Background ("KV cache and
 *       PagedAttention"): K and V of a request live in fixed-size blocks that a
 *       block table maps to physical offsets; the attention itself is the
 *       standard softmax(q K^T / sqrt(D)) V because the balloon driver requires
 *       no change to attention kernels (Sec. 4.2, R4 / D4).
 *
 * Pins (tests, CPU only): dense attention by a library routine on gathered
 * tensors, closed forms (uniform keys -> mean of V, one token -> that V row,
 * dominant key), softmax rows summing to one, invariance under physical
 * placement, e4m3 decode against a library conversion of all 256 codes,
 * conservation / disjointness / LIFO / first-fit properties and an independent
 * list-and-set model of the bookkeeping on small pools.
 */
#define _GNU_SOURCE
#include "prism_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <sys/mman.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_POOLS 8
#define ORC_MAX_MODELS 64
#define ORC_FP8_HEADER 128 /* bytes: fp32 sK[Hkv], fp32 sV[Hkv], padding */
#define ORC_DEFAULT_FRAME ((size_t)2 << 20)
#define ORC_DEFAULT_MAX_SEQS 256
#define ORC_DEFAULT_MAX_BLOCKS 2048

typedef struct {
    int live;
    size_t bytes, frame_bytes;
    int T;              /* tokens per block */
    long n_frames;
    int32_t *owner;     /* model id or -1 */
    uint32_t *free_stack; /* [0] bottom ... [n_free-1] top */
    long n_free;
    uint8_t *mem;       /* mirror of the pool bytes, committed lazily */
    size_t map_len;
} pool_t;

typedef struct {
    int live;
    int pool;
    int Hq, Hkv, D, dtype, g;
    int L, layer;       /* layers sharing one block table; the layer the KV calls address */
    size_t layer_bytes; /* one layer's part of a block */
    size_t block_bytes; /* all layers: L * layer_bytes */
    int slots;          /* blocks per frame */
    long owned;
    uint32_t *frames;   /* acquisition order */
    uint8_t *used;      /* one byte per slot, frame-major: used[i*slots + s] */
    int max_seqs, max_blocks;
    int32_t *rows;      /* [max_seqs][max_blocks] physical block ids */
    int32_t *row_len;
} model_t;

static pool_t g_pools[ORC_MAX_POOLS];
static model_t g_models[ORC_MAX_MODELS];

static pool_t *get_pool(int id) {
    if (id < 0 || id >= ORC_MAX_POOLS || !g_pools[id].live) return NULL;
    return &g_pools[id];
}
static model_t *get_model(int id) {
    if (id < 0 || id >= ORC_MAX_MODELS || !g_models[id].live) return NULL;
    return &g_models[id];
}

/* ------------------------------------------------------------------ pool */

int orc_pool_create_ex(size_t bytes, int page_tokens, size_t frame_bytes) {
    if (page_tokens <= 0 || frame_bytes == 0 || bytes < frame_bytes) return ORC_E_ARG;
    int id = -1;
    for (int i = 0; i < ORC_MAX_POOLS; ++i)
        if (!g_pools[i].live) { id = i; break; }
    if (id < 0) return ORC_E_NOMEM;
    pool_t *p = &g_pools[id];
    memset(p, 0, sizeof *p);
    p->bytes = bytes;
    p->frame_bytes = frame_bytes;
    p->T = page_tokens;
    p->n_frames = (long)(bytes / frame_bytes);
    if (p->n_frames > 0x7fffffffL / 4) return ORC_E_ARG;
    p->owner = malloc(sizeof(int32_t) * (size_t)p->n_frames);
    p->free_stack = malloc(sizeof(uint32_t) * (size_t)p->n_frames);
    p->map_len = (size_t)p->n_frames * frame_bytes;
    p->mem = mmap(NULL, p->map_len, PROT_READ | PROT_WRITE,
                  MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
    if (!p->owner || !p->free_stack || p->mem == MAP_FAILED) {
        free(p->owner); free(p->free_stack);
        if (p->mem != MAP_FAILED) munmap(p->mem, p->map_len);
        return ORC_E_NOMEM;
    }
    for (long f = 0; f < p->n_frames; ++f) {
        p->owner[f] = -1;
        /* top of the stack is the last element: pops hand out 0, 1, 2, ... */
        p->free_stack[f] = (uint32_t)(p->n_frames - 1 - f);
    }
    p->n_free = p->n_frames;
    p->live = 1;
    return id;
}

int orc_pool_create(size_t bytes, int page_tokens) {
    return orc_pool_create_ex(bytes, page_tokens, ORC_DEFAULT_FRAME);
}

int orc_pool_destroy(int pool) {
    pool_t *p = get_pool(pool);
    if (!p) return ORC_E_HANDLE;
    for (int m = 0; m < ORC_MAX_MODELS; ++m)
        if (g_models[m].live && g_models[m].pool == pool) return ORC_E_BUSY;
    free(p->owner);
    free(p->free_stack);
    munmap(p->mem, p->map_len);
    p->live = 0;
    return ORC_OK;
}

/* perm lists the frames in the order pops shall hand them out. */
int orc_pool_seed_free_order(int pool, const uint32_t *perm, size_t n) {
    pool_t *p = get_pool(pool);
    if (!p) return ORC_E_HANDLE;
    if (!perm || (long)n != p->n_frames || p->n_free != p->n_frames) return ORC_E_ARG;
    uint8_t *seen = calloc((size_t)p->n_frames, 1);
    if (!seen) return ORC_E_NOMEM;
    for (size_t i = 0; i < n; ++i) {
        if (perm[i] >= (uint32_t)p->n_frames || seen[perm[i]]) { free(seen); return ORC_E_ARG; }
        seen[perm[i]] = 1;
    }
    free(seen);
    for (size_t i = 0; i < n; ++i) p->free_stack[n - 1 - i] = perm[i];
    return ORC_OK;
}

/* ----------------------------------------------------------------- model */

/* Sec. 4.2, D3 (first optimisation): a model of L layers keeps the K and V of all its
 * layers for one token block side by side, so one block id, one slot and one block-table
 * row serve every layer, and a reserve is one allocation instead of 2L.  Here a block is
 * L consecutive layer parts; the part of layer l starts l * layer_bytes into the block. */
int orc_model_register_layers(int pool, int q_heads, int kv_heads, int head_dim, int dtype,
                              int max_seqs, int max_blocks_per_seq, int n_layers) {
    pool_t *p = get_pool(pool);
    if (!p) return ORC_E_HANDLE;
    if (q_heads <= 0 || kv_heads <= 0 || head_dim <= 0 || max_seqs <= 0 || max_blocks_per_seq <= 0 ||
        n_layers <= 0)
        return ORC_E_ARG;
    if (dtype != ORC_BF16 && dtype != ORC_E4M3) return ORC_E_ARG;
    if (q_heads % kv_heads != 0) return ORC_E_SHAPE;
    size_t e = dtype == ORC_BF16 ? 2 : 1;
    size_t block_bytes = (size_t)2 * (size_t)p->T * (size_t)kv_heads * (size_t)head_dim * e;
    if (dtype == ORC_E4M3) {
        if ((size_t)kv_heads * 2 * sizeof(float) > ORC_FP8_HEADER) return ORC_E_SHAPE;
        block_bytes += ORC_FP8_HEADER;
    }
    const size_t layer_bytes = block_bytes;
    block_bytes *= (size_t)n_layers;
    size_t slots = p->frame_bytes / block_bytes;
    if (slots == 0) return ORC_E_SHAPE;
    int id = -1;
    for (int i = 0; i < ORC_MAX_MODELS; ++i)
        if (!g_models[i].live) { id = i; break; }
    if (id < 0) return ORC_E_NOMEM;
    model_t *m = &g_models[id];
    memset(m, 0, sizeof *m);
    m->pool = pool;
    m->Hq = q_heads; m->Hkv = kv_heads; m->D = head_dim; m->dtype = dtype;
    m->g = q_heads / kv_heads;
    m->L = n_layers;
    m->layer = 0;
    m->layer_bytes = layer_bytes;
    m->block_bytes = block_bytes;
    m->slots = (int)slots;
    m->max_seqs = max_seqs;
    m->max_blocks = max_blocks_per_seq;
    m->rows = calloc((size_t)max_seqs * (size_t)max_blocks_per_seq, sizeof(int32_t));
    m->row_len = calloc((size_t)max_seqs, sizeof(int32_t));
    if (!m->rows || !m->row_len) { free(m->rows); free(m->row_len); return ORC_E_NOMEM; }
    m->live = 1;
    return id;
}

int orc_model_register_ex(int pool, int q_heads, int kv_heads, int head_dim, int dtype,
                          int max_seqs, int max_blocks_per_seq) {
    return orc_model_register_layers(pool, q_heads, kv_heads, head_dim, dtype, max_seqs, max_blocks_per_seq, 1);
}

/* the layer that kv_write / kv_append / kv_read and the attention calls address from now on */
int orc_set_layer(int model, int layer) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (layer < 0 || layer >= m->L) return ORC_E_ARG;
    m->layer = layer;
    return ORC_OK;
}

int orc_model_register(int pool, int q_heads, int kv_heads, int head_dim, int dtype) {
    return orc_model_register_ex(pool, q_heads, kv_heads, head_dim, dtype,
                                 ORC_DEFAULT_MAX_SEQS, ORC_DEFAULT_MAX_BLOCKS);
}

int orc_model_unregister(int model) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (m->owned != 0) return ORC_E_BUSY;
    free(m->frames); free(m->used); free(m->rows); free(m->row_len);
    m->live = 0;
    return ORC_OK;
}

/* --------------------------------------------------------------- balloon */

static int frame_is_empty(const model_t *m, long i) {
    for (int s = 0; s < m->slots; ++s)
        if (m->used[(size_t)i * m->slots + s]) return 0;
    return 1;
}

long orc_balloon_resize(int model, long target) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (target < 0) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    if (target > m->owned) {
        /* inflate: all or nothing */
        long need = target - m->owned;
        if (need > p->n_free) return ORC_E_NOMEM;
        uint32_t *nf = realloc(m->frames, sizeof(uint32_t) * (size_t)target);
        if (!nf) return ORC_E_INTERNAL;
        m->frames = nf;
        uint8_t *nu = realloc(m->used, (size_t)target * m->slots);
        if (!nu) return ORC_E_INTERNAL;
        m->used = nu;
        for (long k = 0; k < need; ++k) {
            uint32_t f = p->free_stack[--p->n_free];      /* pop */
            p->owner[f] = model;
            m->frames[m->owned] = f;                       /* append */
            memset(m->used + (size_t)m->owned * m->slots, 0, (size_t)m->slots);
            m->owned++;
        }
        return m->owned;
    }
    if (target < m->owned) {
        /* deflate: give back empty frames, newest first, until the target is
         * met; frames that still hold blocks stay (clamp). */
        long want = m->owned - target, reclaimed = 0;
        uint8_t *mark = calloc((size_t)m->owned, 1);
        if (!mark) return ORC_E_INTERNAL;
        for (long i = m->owned - 1; i >= 0 && reclaimed < want; --i) {
            if (frame_is_empty(m, i)) {
                mark[i] = 1;
                uint32_t f = m->frames[i];
                p->free_stack[p->n_free++] = f;            /* push in scan order */
                p->owner[f] = -1;
                reclaimed++;
            }
        }
        long w = 0; /* delete marked entries, keep the order of the rest */
        for (long i = 0; i < m->owned; ++i) {
            if (mark[i]) continue;
            if (w != i) {
                m->frames[w] = m->frames[i];
                memmove(m->used + (size_t)w * m->slots, m->used + (size_t)i * m->slots,
                        (size_t)m->slots);
            }
            w++;
        }
        m->owned = w;
        free(mark);
        return m->owned;
    }
    return m->owned;
}

/* ------------------------------------------------------------ block rows */

static long blocks_for(const pool_t *p, int ctx_len) {
    return ((long)ctx_len + p->T - 1) / p->T;
}

static long free_slots(const model_t *m) {
    long z = 0;
    for (long j = 0; j < m->owned * m->slots; ++j) z += !m->used[j];
    return z;
}

/* append `need` blocks to a row: lowest-index free slots first */
static void place_blocks(model_t *m, int seq, long need) {
    long j = 0;
    while (need > 0) {
        while (m->used[j]) ++j;
        m->used[j] = 1;
        int32_t block_id = (int32_t)((long)m->frames[j / m->slots] * m->slots + (j % m->slots));
        m->rows[(size_t)seq * m->max_blocks + m->row_len[seq]] = block_id;
        m->row_len[seq]++;
        --need;
    }
}

int orc_seq_reserve(int model, int seq, int ctx_len) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (seq < 0 || seq >= m->max_seqs || ctx_len < 0) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    long want = blocks_for(p, ctx_len);
    if (want > m->max_blocks) return ORC_E_RANGE;
    long need = want - m->row_len[seq];
    if (need <= 0) return 0;
    if (need > free_slots(m)) return ORC_E_BALLOON;
    place_blocks(m, seq, need);
    return (int)need;
}

/* same result as calling orc_seq_reserve for each entry in order, except that
 * the whole batch is refused (nothing changes) when it does not fit. */
int orc_seq_reserve_batch(int model, int n, const int32_t *seqs, const int32_t *ctx_lens) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (n < 0 || (n > 0 && (!seqs || !ctx_lens))) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    int32_t *len = malloc(sizeof(int32_t) * (size_t)m->max_seqs);
    if (!len) return ORC_E_INTERNAL;
    memcpy(len, m->row_len, sizeof(int32_t) * (size_t)m->max_seqs);
    long total = 0;
    for (int i = 0; i < n; ++i) {
        if (seqs[i] < 0 || seqs[i] >= m->max_seqs || ctx_lens[i] < 0) { free(len); return ORC_E_ARG; }
        long want = blocks_for(p, ctx_lens[i]);
        if (want > m->max_blocks) { free(len); return ORC_E_RANGE; }
        if (want > len[seqs[i]]) { total += want - len[seqs[i]]; len[seqs[i]] = (int32_t)want; }
    }
    free(len);
    if (total > free_slots(m)) return ORC_E_BALLOON;
    for (int i = 0; i < n; ++i) {
        long need = blocks_for(p, ctx_lens[i]) - m->row_len[seqs[i]];
        if (need > 0) place_blocks(m, seqs[i], need);
    }
    return (int)total;
}

int orc_seq_release(int model, int seq) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (seq < 0 || seq >= m->max_seqs) return ORC_E_ARG;
    int n = m->row_len[seq];
    for (int b = 0; b < n; ++b) {
        int32_t id = m->rows[(size_t)seq * m->max_blocks + b];
        uint32_t f = (uint32_t)(id / m->slots);
        long i = 0;
        while (i < m->owned && m->frames[i] != f) ++i;   /* position of the frame */
        if (i == m->owned) return ORC_E_INTERNAL;
        m->used[(size_t)i * m->slots + (id % m->slots)] = 0;
    }
    m->row_len[seq] = 0;
    return n;
}

/* -------------------------------------------------------- addressing, KV */

/* byte offset, inside the pool, of the current layer's part of a block */
static size_t block_addr(const model_t *m, const pool_t *p, int32_t block_id) {
    return (size_t)(block_id / m->slots) * p->frame_bytes +
           (size_t)(block_id % m->slots) * m->block_bytes +
           (size_t)m->layer * m->layer_bytes;
}

/* in-block layout: [e4m3 only: 128 B header] then [kvh][K|V][token slot][d] */
static size_t elem_index(const model_t *m, const pool_t *p, int kvh, int which, int slot, int d) {
    if (kvh < 0 || kvh >= m->Hkv) return 0;
    return (((size_t)kvh * 2 + (size_t)which) * (size_t)p->T + (size_t)slot) * (size_t)m->D + (size_t)d;
}

static double bf16_to_double(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3 (finite-only variant): sign, 4 exponent bits with bias 7,
 * 3 mantissa bits; exponent 0 is subnormal; S.1111.111 is NaN; no infinities. */
double orc_e4m3_decode(uint8_t c) {
    int s = c >> 7, E = (c >> 3) & 15, M = c & 7;
    double v;
    if (E == 15 && M == 7) return NAN;
    if (E == 0) v = ldexp((double)M / 8.0, -6);
    else v = ldexp(1.0 + (double)M / 8.0, E - 7);
    return s ? -v : v;
}

static double kv_value(const model_t *m, const pool_t *p, int32_t block_id, int kvh, int which,
                       int slot, int d) {
    const uint8_t *blk = p->mem + block_addr(m, p, block_id);
    size_t i = elem_index(m, p, kvh, which, slot, d);
    if (m->dtype == ORC_BF16) {
        uint16_t b;
        memcpy(&b, blk + i * 2, 2);
        return bf16_to_double(b);
    }
    float scale;
    memcpy(&scale, blk + sizeof(float) * ((size_t)which * m->Hkv + kvh), sizeof scale);
    return orc_e4m3_decode(blk[ORC_FP8_HEADER + i]) * (double)scale;
}

int orc_kv_write(int model, int seq, int tok_begin, int n_tok, const void *k, const void *v,
                 const float *k_scale, const float *v_scale) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (seq < 0 || seq >= m->max_seqs || tok_begin < 0 || n_tok < 0) return ORC_E_ARG;
    if (n_tok == 0) return 0;
    if (!k || !v) return ORC_E_ARG;
    if (m->dtype == ORC_E4M3 && (!k_scale || !v_scale)) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    if (((long)tok_begin + n_tok + p->T - 1) / p->T > m->row_len[seq]) return ORC_E_RANGE;
    size_t e = m->dtype == ORC_BF16 ? 2 : 1;
    size_t hdr = m->dtype == ORC_E4M3 ? ORC_FP8_HEADER : 0;
    int first_blk = tok_begin / p->T;
    for (int t = 0; t < n_tok; ++t) {
        int tok = tok_begin + t;
        int32_t id = m->rows[(size_t)seq * m->max_blocks + tok / p->T];
        uint8_t *blk = p->mem + block_addr(m, p, id);
        for (int h = 0; h < m->Hkv; ++h) {
            size_t src = ((size_t)t * m->Hkv + h) * m->D * e;
            memcpy(blk + hdr + elem_index(m, p, h, 0, tok % p->T, 0) * e, (const uint8_t *)k + src, m->D * e);
            memcpy(blk + hdr + elem_index(m, p, h, 1, tok % p->T, 0) * e, (const uint8_t *)v + src, m->D * e);
            if (m->dtype == ORC_E4M3) {
                size_t si = (size_t)(tok / p->T - first_blk) * m->Hkv + h;
                memcpy(blk + sizeof(float) * (size_t)h, &k_scale[si], sizeof(float));
                memcpy(blk + sizeof(float) * ((size_t)m->Hkv + h), &v_scale[si], sizeof(float));
            }
        }
    }
    return n_tok;
}

/* Nearest E4M3 value of y, ties to the even code, magnitudes beyond the largest
 * finite value (448) saturating to it: written out as a search over the 127 finite
 * magnitudes, whose values are exact in double. */
uint8_t orc_e4m3_encode(float y) {
    if (y != y) return 0x7F;
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    double a = fabs((double)y);
    if (a >= 448.0) return (uint8_t)(sign | 0x7E);
    int best = 0;
    double best_err = a;                         /* code 0 is +0 */
    for (int c = 1; c <= 0x7E; ++c) {
        double err = fabs(orc_e4m3_decode((uint8_t)c) - a);
        if (err < best_err || (err == best_err && (c & 1) == 0)) { best = c; best_err = err; }
    }
    return (uint8_t)(sign | best);
}

/* The write path of a decode step (paper: Sec. 4.2 D2, a sequence that grows takes its
 * next token block from the slots of its pages; the new token's K and V are scattered
 * into that block).  For every sequence s of the batch the token with index
 * ctx_lens[s] - 1 is written; k_new, v_new are bf16 bit patterns [batch][Hkv][D].
 *
 * bf16 models store the values as they are.  e4m3 models keep one fp32 scale per (block,
 * kv head) for K and one for V, equal to the running maximum of amax / 448 over the
 * block's tokens, all arithmetic in fp32:
 *   slot 0 of a block:   scale = amax > 0 ? amax / 448 : 1
 *   later slots:         cand = amax / 448; if cand > scale, every code c already in the
 *                        block becomes encode((decode(c) * scale) / cand) and scale = cand
 *   the new token:       code = encode(x / scale)
 * where amax = max_d |x[d]| of the token's row for that kv head. */
static void append_row_e4m3(const model_t *m, const pool_t *p, uint8_t *blk, int kvh, int which, int slot,
                            const uint16_t *x_bf16) {
    float *scale_p = (float *)(blk + sizeof(float) * ((size_t)which * m->Hkv + kvh));
    uint8_t *codes = blk + ORC_FP8_HEADER;
    float amax = 0.0f;
    for (int d = 0; d < m->D; ++d) {
        float x = (float)bf16_to_double(x_bf16[d]);
        if (fabsf(x) > amax) amax = fabsf(x);
    }
    float cand = amax / 448.0f;
    float scale;
    if (slot == 0) {
        scale = amax > 0.0f ? cand : 1.0f;
    } else {
        memcpy(&scale, scale_p, sizeof scale);
        if (cand > scale) {
            for (int t = 0; t < slot; ++t)
                for (int d = 0; d < m->D; ++d) {
                    uint8_t *c = &codes[elem_index(m, p, kvh, which, t, d)];
                    float v = (float)orc_e4m3_decode(*c) * scale;     /* fp32 product */
                    *c = orc_e4m3_encode(v / cand);                    /* fp32 quotient */
                }
            scale = cand;
        }
    }
    memcpy(scale_p, &scale, sizeof scale);
    for (int d = 0; d < m->D; ++d) {
        float x = (float)bf16_to_double(x_bf16[d]);
        codes[elem_index(m, p, kvh, which, slot, d)] = orc_e4m3_encode(x / scale);
    }
}

/* one token of sequence s at index tok; kx, vx: [Hkv][D] */
static void append_token(const model_t *m, const pool_t *p, int s, int tok, const uint16_t *kx, const uint16_t *vx) {
    int slot = tok % p->T;
    int32_t id = m->rows[(size_t)s * m->max_blocks + tok / p->T];
    uint8_t *blk = p->mem + block_addr(m, p, id);
    for (int h = 0; h < m->Hkv; ++h) {
        const uint16_t *kh = kx + (size_t)h * m->D, *vh = vx + (size_t)h * m->D;
        if (m->dtype == ORC_BF16) {
            memcpy(blk + elem_index(m, p, h, 0, slot, 0) * 2, kh, (size_t)m->D * 2);
            memcpy(blk + elem_index(m, p, h, 1, slot, 0) * 2, vh, (size_t)m->D * 2);
        } else {
            append_row_e4m3(m, p, blk, h, 0, slot, kh);
            append_row_e4m3(m, p, blk, h, 1, slot, vh);
        }
    }
}

int orc_kv_append(int model, int batch, const uint16_t *k_new, const uint16_t *v_new, const int32_t *ctx_lens) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (batch < 0 || batch > m->max_seqs) return ORC_E_RANGE;
    if (batch == 0) return 0;
    if (!k_new || !v_new || !ctx_lens) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    for (int s = 0; s < batch; ++s)
        if (ctx_lens[s] < 1 || blocks_for(p, ctx_lens[s]) > m->row_len[s]) return ORC_E_RANGE;
    for (int s = 0; s < batch; ++s)
        append_token(m, p, s, ctx_lens[s] - 1, k_new + (size_t)s * m->Hkv * m->D, v_new + (size_t)s * m->Hkv * m->D);
    return batch;
}

/* The write path of a prefill chunk: sequence s appends its q_lens[s] new tokens, packed one
 * sequence after the other in k_new, v_new [sum q_lens][Hkv][D], at the indices
 * ctx_lens[s] - q_lens[s] .. ctx_lens[s] - 1.  Defined as orc_kv_append applied token by
 * token in order, so a cache filled in chunks equals one filled a token at a time. */
int orc_kv_append_chunk(int model, int batch, const uint16_t *k_new, const uint16_t *v_new, const int32_t *q_lens,
                        const int32_t *ctx_lens) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (batch < 0 || batch > m->max_seqs) return ORC_E_RANGE;
    if (batch == 0) return 0;
    if (!k_new || !v_new || !q_lens || !ctx_lens) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    long total = 0;
    for (int s = 0; s < batch; ++s) {
        if (q_lens[s] < 0) return ORC_E_ARG;
        if (q_lens[s] > 0 && (ctx_lens[s] < q_lens[s] || blocks_for(p, ctx_lens[s]) > m->row_len[s])) return ORC_E_RANGE;
        total += q_lens[s];
    }
    size_t row = 0;
    for (int s = 0; s < batch; ++s)
        for (int i = 0; i < q_lens[s]; ++i, ++row)
            append_token(m, p, s, ctx_lens[s] - q_lens[s] + i, k_new + row * m->Hkv * m->D, v_new + row * m->Hkv * m->D);
    return (int)total;
}

/* Read tokens back in the logical layout of orc_kv_write: k_out, v_out [n_tok][Hkv][D]
 * elements; e4m3 only: k_scale_out, v_scale_out fp32 [n_tok][Hkv], the scale of the block
 * each token lives in. */
int orc_kv_read(int model, int seq, int tok_begin, int n_tok, void *k_out, void *v_out,
                float *k_scale_out, float *v_scale_out) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (seq < 0 || seq >= m->max_seqs || tok_begin < 0 || n_tok < 0) return ORC_E_ARG;
    if (n_tok == 0) return 0;
    if (!k_out || !v_out) return ORC_E_ARG;
    if (m->dtype == ORC_E4M3 && (!k_scale_out || !v_scale_out)) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    if (((long)tok_begin + n_tok + p->T - 1) / p->T > m->row_len[seq]) return ORC_E_RANGE;
    size_t e = m->dtype == ORC_BF16 ? 2 : 1;
    size_t hdr = m->dtype == ORC_E4M3 ? ORC_FP8_HEADER : 0;
    for (int t = 0; t < n_tok; ++t) {
        int tok = tok_begin + t;
        int32_t id = m->rows[(size_t)seq * m->max_blocks + tok / p->T];
        const uint8_t *blk = p->mem + block_addr(m, p, id);
        for (int h = 0; h < m->Hkv; ++h) {
            size_t dst = ((size_t)t * m->Hkv + h) * m->D * e;
            memcpy((uint8_t *)k_out + dst, blk + hdr + elem_index(m, p, h, 0, tok % p->T, 0) * e, m->D * e);
            memcpy((uint8_t *)v_out + dst, blk + hdr + elem_index(m, p, h, 1, tok % p->T, 0) * e, m->D * e);
            if (m->dtype == ORC_E4M3) {
                memcpy(&k_scale_out[(size_t)t * m->Hkv + h], blk + sizeof(float) * (size_t)h, sizeof(float));
                memcpy(&v_scale_out[(size_t)t * m->Hkv + h], blk + sizeof(float) * ((size_t)m->Hkv + h), sizeof(float));
            }
        }
    }
    return n_tok;
}

/* ------------------------------------------------------------- attention */

static int check_row(const model_t *m, const pool_t *p, const int32_t *row, int ctx_len) {
    long nb = blocks_for(p, ctx_len);
    for (long b = 0; b < nb; ++b)
        if (row[b] < 0 || (long)row[b] >= p->n_frames * (long)m->slots) return ORC_E_RANGE;
    return ORC_OK;
}

/* softmax row of one (sequence, q head):
 *   z[t] = (q . k[t]) / sqrt(D),  p[t] = exp(z[t] - max z) / sum_t exp(z[t] - max z) */
static void softmax_row(const model_t *m, const pool_t *p, const uint16_t *q_row,
                        const int32_t *row, int L, int kvh, double *pr) {
    for (int t = 0; t < L; ++t) {
        double dot = 0.0;
        for (int d = 0; d < m->D; ++d)
            dot += bf16_to_double(q_row[d]) * kv_value(m, p, row[t / p->T], kvh, 0, t % p->T, d);
        pr[t] = dot / sqrt((double)m->D);
    }
    double zmax = pr[0];
    for (int t = 1; t < L; ++t) if (pr[t] > zmax) zmax = pr[t];
    double denom = 0.0;
    for (int t = 0; t < L; ++t) { pr[t] = exp(pr[t] - zmax); denom += pr[t]; }
    for (int t = 0; t < L; ++t) pr[t] /= denom;
}

int orc_attention_probs(int model, const uint16_t *q_row, const int32_t *table_row, int ctx_len,
                        int q_head, double *p_out) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (!q_row || !table_row || !p_out || ctx_len <= 0 || q_head < 0 || q_head >= m->Hq) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    if (check_row(m, p, table_row, ctx_len)) return ORC_E_RANGE;
    softmax_row(m, p, q_row, table_row, ctx_len, q_head / m->g, p_out);
    return ORC_OK;
}

int orc_decode_attention(int model, int batch, const uint16_t *q, const int32_t *block_table,
                         int row_stride, const int32_t *ctx_lens, float *out) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (batch < 0 || (batch > 0 && (!q || !ctx_lens || !out))) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    if (!block_table) {
        if (batch > m->max_seqs) return ORC_E_RANGE;
        block_table = m->rows;
        row_stride = m->max_blocks;
        for (int s = 0; s < batch; ++s)
            if (blocks_for(p, ctx_lens[s]) > m->row_len[s]) return ORC_E_RANGE;
    }
    for (int s = 0; s < batch; ++s) {
        if (ctx_lens[s] < 0 || blocks_for(p, ctx_lens[s]) > row_stride) return ORC_E_RANGE;
        if (check_row(m, p, block_table + (size_t)s * row_stride, ctx_lens[s])) return ORC_E_RANGE;
    }
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < batch; ++s) {
        for (int h = 0; h < m->Hq; ++h) {
            const int32_t *row = block_table + (size_t)s * row_stride;
            const uint16_t *q_row = q + ((size_t)s * m->Hq + h) * m->D;
            float *o = out + ((size_t)s * m->Hq + h) * m->D;
            int L = ctx_lens[s];
            int kvh = h / m->g;                 /* contiguous groups of g query heads */
            if (L == 0) { for (int d = 0; d < m->D; ++d) o[d] = 0.0f; continue; }
            double *pr = malloc(sizeof(double) * (size_t)L);
            if (!pr) { failed = 1; continue; }
            softmax_row(m, p, q_row, row, L, kvh, pr);
            for (int d = 0; d < m->D; ++d) {
                double acc = 0.0;
                for (int t = 0; t < L; ++t)
                    acc += pr[t] * kv_value(m, p, row[t / p->T], kvh, 1, t % p->T, d);
                o[d] = (float)acc;
            }
            free(pr);
        }
    }
    return failed ? ORC_E_INTERNAL : ORC_OK;
}

/* Causal attention of a chunk of new tokens against the paged cache (paper: Sec. 5.2,
 * prefill proceeds in chunks, every chunk attending to the cache built so far).  Sequence
 * s brings q_lens[s] queries, packed one sequence after the other in q [sum q_lens][Hq][D];
 * its cache already holds ctx_lens[s] tokens, the chunk's own included.  Query i of the
 * sequence stands at position pos = ctx_lens[s] - q_lens[s] + i and sees the tokens
 * t <= pos:   out = softmax_t<=pos(q . k[t] / sqrt(D)) V,   fp64, stored as fp32
 * [sum q_lens][Hq][D]. */
int orc_prefill_attention(int model, int batch, const uint16_t *q, const int32_t *q_lens,
                          const int32_t *block_table, int row_stride, const int32_t *ctx_lens, float *out) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (batch < 0 || (batch > 0 && (!q || !q_lens || !ctx_lens || !out))) return ORC_E_ARG;
    pool_t *p = &g_pools[m->pool];
    if (!block_table) {
        if (batch > m->max_seqs) return ORC_E_RANGE;
        block_table = m->rows;
        row_stride = m->max_blocks;
        for (int s = 0; s < batch; ++s)
            if (blocks_for(p, ctx_lens[s]) > m->row_len[s]) return ORC_E_RANGE;
    }
    long total_q = 0;
    for (int s = 0; s < batch; ++s) {
        if (q_lens[s] < 0 || ctx_lens[s] < q_lens[s] || blocks_for(p, ctx_lens[s]) > row_stride) return ORC_E_RANGE;
        if (check_row(m, p, block_table + (size_t)s * row_stride, ctx_lens[s])) return ORC_E_RANGE;
        total_q += q_lens[s];
    }
    /* one flat list of (sequence, query) so that the rows can be shared out evenly */
    int32_t *seq_of = malloc(sizeof(int32_t) * (size_t)(total_q > 0 ? total_q : 1));
    int32_t *idx_of = malloc(sizeof(int32_t) * (size_t)(total_q > 0 ? total_q : 1));
    if (!seq_of || !idx_of) { free(seq_of); free(idx_of); return ORC_E_INTERNAL; }
    long r = 0;
    for (int s = 0; s < batch; ++s)
        for (int i = 0; i < q_lens[s]; ++i) { seq_of[r] = s; idx_of[r] = i; ++r; }
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long row_i = 0; row_i < total_q; ++row_i) {
        for (int h = 0; h < m->Hq; ++h) {
            int s = seq_of[row_i];
            int L = ctx_lens[s] - q_lens[s] + idx_of[row_i] + 1;      /* tokens this query sees */
            const int32_t *row = block_table + (size_t)s * row_stride;
            const uint16_t *q_row = q + ((size_t)row_i * m->Hq + h) * m->D;
            float *o = out + ((size_t)row_i * m->Hq + h) * m->D;
            int kvh = h / m->g;
            double *pr = malloc(sizeof(double) * (size_t)L);
            if (!pr) { failed = 1; continue; }
            softmax_row(m, p, q_row, row, L, kvh, pr);
            for (int d = 0; d < m->D; ++d) {
                double acc = 0.0;
                for (int t = 0; t < L; ++t)
                    acc += pr[t] * kv_value(m, p, row[t / p->T], kvh, 1, t % p->T, d);
                o[d] = (float)acc;
            }
            free(pr);
        }
    }
    free(seq_of);
    free(idx_of);
    return failed ? ORC_E_INTERNAL : ORC_OK;
}

/* ---------------------------------------------------------- state export */

typedef struct { int32_t *w; size_t cap, n; } wr_t;
static void put(wr_t *o, long v) {
    if (o->w && o->n < o->cap) o->w[o->n] = (int32_t)v;
    o->n++;
}

long orc_pool_export_state(int pool, void *buf, size_t cap) {
    pool_t *p = get_pool(pool);
    if (!p) return ORC_E_HANDLE;
    /* pass 1 counts, pass 2 writes (only when the buffer is large enough) */
    wr_t o = { NULL, 0, 0 };
    for (int pass = 0; pass < 2; ++pass) {
        o.n = 0;
        put(&o, 0x53564B50);            /* "PKVS" */
        put(&o, 1);                     /* format version */
        put(&o, p->n_frames);
        put(&o, p->T);
        put(&o, p->n_free);
        for (long i = 0; i < p->n_free; ++i) put(&o, (long)p->free_stack[i]);
        for (long f = 0; f < p->n_frames; ++f) put(&o, p->owner[f]);
        long n_models = 0;
        for (int id = 0; id < ORC_MAX_MODELS; ++id)
            if (g_models[id].live && g_models[id].pool == pool) n_models++;
        put(&o, n_models);
        for (int id = 0; id < ORC_MAX_MODELS; ++id) {
            const model_t *m = &g_models[id];
            if (!m->live || m->pool != pool) continue;
            put(&o, id); put(&o, m->Hq); put(&o, m->Hkv); put(&o, m->D); put(&o, m->dtype);
            put(&o, m->slots); put(&o, m->owned);
            for (long i = 0; i < m->owned; ++i) put(&o, (long)m->frames[i]);
            long nbits = m->owned * m->slots;
            put(&o, nbits);
            for (long w = 0; w < (nbits + 31) / 32; ++w) {
                uint32_t word = 0;
                for (int b = 0; b < 32 && w * 32 + b < nbits; ++b)
                    if (m->used[w * 32 + b]) word |= 1u << b;
                put(&o, (long)(int32_t)word);
            }
            put(&o, m->max_seqs);
            long n_rows = 0;
            for (int s = 0; s < m->max_seqs; ++s) n_rows += m->row_len[s] > 0;
            put(&o, n_rows);
            for (int s = 0; s < m->max_seqs; ++s) {
                if (m->row_len[s] == 0) continue;
                put(&o, s); put(&o, m->row_len[s]);
                for (int b = 0; b < m->row_len[s]; ++b) put(&o, m->rows[(size_t)s * m->max_blocks + b]);
            }
        }
        if (pass == 0) {
            if (!buf || cap < o.n * sizeof(int32_t)) return (long)(o.n * sizeof(int32_t));
            o.w = buf; o.cap = cap / sizeof(int32_t);
        }
    }
    return (long)(o.n * sizeof(int32_t));
}

/* --------------------------------------------------------- introspection */

long orc_pool_n_frames(int pool) { pool_t *p = get_pool(pool); return p ? p->n_frames : ORC_E_HANDLE; }
long orc_pool_n_free(int pool) { pool_t *p = get_pool(pool); return p ? p->n_free : ORC_E_HANDLE; }
long orc_model_owned(int model) { model_t *m = get_model(model); return m ? m->owned : ORC_E_HANDLE; }
int orc_model_slots(int model) { model_t *m = get_model(model); return m ? m->slots : ORC_E_HANDLE; }
long orc_model_block_bytes(int model) { model_t *m = get_model(model); return m ? (long)m->block_bytes : ORC_E_HANDLE; }
int orc_model_layers(int model) { model_t *m = get_model(model); return m ? m->L : ORC_E_HANDLE; }
long orc_block_address(int model, int block_id) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    return (long)block_addr(m, &g_pools[m->pool], block_id);
}
const int32_t *orc_model_block_table(int model, int *row_stride) {
    model_t *m = get_model(model);
    if (!m) return NULL;
    if (row_stride) *row_stride = m->max_blocks;
    return m->rows;
}
int orc_model_row_len(int model, int seq) {
    model_t *m = get_model(model);
    if (!m) return ORC_E_HANDLE;
    if (seq < 0 || seq >= m->max_seqs) return ORC_E_ARG;
    return m->row_len[seq];
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
