/*
 * prism_oracle.h — CPU oracle for the shared-pool paged decode attention path.
 *
 * TEST INFRASTRUCTURE ONLY.  This library is the slow, plain definition that the
 * GPU library is checked against.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may load it; the product library never does and
 * shares no source, header, table or helper with it.
 *
 * What it defines (paper: Background, "KV cache and PagedAttention"; Sec. 4.2,
 * designs D1-D3 of the balloon driver):
 *   - one physical pool cut into fixed-size frames; a frame is owned by at most
 *     one model (D2: blocks of different models live on distinct pages);
 *   - a model's balloon = the frames it owns; balloon_resize moves frames between
 *     the pool's free stack and the model (D1: limits shrink and grow; memory is
 *     only reassigned, never created);
 *   - token blocks are placed first-fit into slots of the model's frames
 *     (D2/D3: slots inside a page, partially filled pages first);
 *   - decode attention out = softmax(q K^T / sqrt(D)) V over the tokens a
 *     sequence's block-table row addresses, in fp64, stored as fp32.
 *
 * Every function returns 0 / a non-negative count on success and a negative
 * ORC_E_* code on error.  A failing call leaves the state untouched.
 * All pointers are host pointers.
 */
#ifndef PRISM_ORACLE_H
#define PRISM_ORACLE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ORC_OK = 0,
    ORC_E_ARG = -1,      /* bad argument value */
    ORC_E_HANDLE = -2,   /* unknown pool / model id */
    ORC_E_NOMEM = -3,    /* inflate: not enough free frames (state unchanged) */
    ORC_E_BALLOON = -4,  /* reserve: not enough free slots in the balloon */
    ORC_E_SHAPE = -5,    /* block does not fit a frame, Hq % Hkv != 0, ... */
    ORC_E_RANGE = -6,    /* index outside table / pool / buffer too small */
    ORC_E_BUSY = -7,     /* destroy / unregister while frames are owned */
    ORC_E_INTERNAL = -8
};

enum { ORC_BF16 = 0, ORC_E4M3 = 1 };

int orc_pool_create(size_t bytes, int page_tokens); /* frame_bytes = 2 MiB */
int orc_pool_create_ex(size_t bytes, int page_tokens, size_t frame_bytes);
int orc_pool_destroy(int pool);
int orc_pool_seed_free_order(int pool, const uint32_t *perm, size_t n);

int orc_model_register(int pool, int q_heads, int kv_heads, int head_dim, int dtype);
int orc_model_register_ex(int pool, int q_heads, int kv_heads, int head_dim, int dtype,
                          int max_seqs, int max_blocks_per_seq);
/* a model of n_layers layers: every block holds all layers' K and V (Sec. 4.2, D3), one
 * block table serves them all; orc_set_layer picks the layer the KV and attention calls address */
int orc_model_register_layers(int pool, int q_heads, int kv_heads, int head_dim, int dtype,
                              int max_seqs, int max_blocks_per_seq, int n_layers);
int orc_set_layer(int model, int layer);
int orc_model_layers(int model);
int orc_model_unregister(int model);

long orc_balloon_resize(int model, long frames);
int orc_seq_reserve(int model, int seq, int ctx_len);
int orc_seq_reserve_batch(int model, int n, const int32_t *seqs, const int32_t *ctx_lens);
int orc_seq_release(int model, int seq);

/* logical k, v: [n_tok][Hkv][D] elements (bf16 bit patterns or e4m3 bytes);
 * e4m3 only: k_scale, v_scale = fp32 [n_blocks_touched][Hkv], first row = the
 * block that holds tok_begin. */
int orc_kv_write(int model, int seq, int tok_begin, int n_tok, const void *k, const void *v,
                 const float *k_scale, const float *v_scale);

/* decode-step write path: the token with index ctx_lens[s] - 1 of every sequence
 * s < batch; k_new, v_new bf16 bit patterns [batch][Hkv][D].  e4m3 models quantise
 * with a running per-(block, kv head) scale (rule stated at the definition). */
int orc_kv_append(int model, int batch, const uint16_t *k_new, const uint16_t *v_new, const int32_t *ctx_lens);
/* a prefill chunk: q_lens[s] tokens per sequence, packed [sum q_lens][Hkv][D], written at
 * ctx_lens[s] - q_lens[s] .. ctx_lens[s] - 1; equals orc_kv_append token by token. */
int orc_kv_append_chunk(int model, int batch, const uint16_t *k_new, const uint16_t *v_new, const int32_t *q_lens,
                        const int32_t *ctx_lens);

/* tokens back in the logical layout of orc_kv_write; e4m3 only: scales per token
 * [n_tok][Hkv] (the scale of the token's block). */
int orc_kv_read(int model, int seq, int tok_begin, int n_tok, void *k_out, void *v_out,
                float *k_scale_out, float *v_scale_out);

/* q: bf16 bit patterns [B][Hq][D]; block_table NULL = the model's own rows 0..B-1
 * (row_stride ignored); out fp32 [B][Hq][D]. */
int orc_decode_attention(int model, int batch, const uint16_t *q, const int32_t *block_table,
                         int row_stride, const int32_t *ctx_lens, float *out);

/* causal attention of a chunk: q [sum q_lens][Hq][D] packed by sequence, the cache
 * holds ctx_lens[s] tokens (the chunk's included), query i of s sees t <= ctx_lens[s]
 * - q_lens[s] + i; out fp32 [sum q_lens][Hq][D]. */
int orc_prefill_attention(int model, int batch, const uint16_t *q, const int32_t *q_lens,
                          const int32_t *block_table, int row_stride, const int32_t *ctx_lens, float *out);

/* debug: the softmax row p[0..ctx_len) of one (sequence, q head), in fp64 */
int orc_attention_probs(int model, const uint16_t *q_row, const int32_t *table_row, int ctx_len,
                        int q_head, double *p_out);

/* canonical little-endian int32 image of the bookkeeping state; returns the byte
 * count needed, writes only when cap is large enough. */
long orc_pool_export_state(int pool, void *buf, size_t cap);

/* introspection used by tests */
long orc_pool_n_frames(int pool);
long orc_pool_n_free(int pool);
long orc_model_owned(int model);
int orc_model_slots(int model);
long orc_model_block_bytes(int model);
long orc_block_address(int model, int block_id); /* byte offset in the pool */
const int32_t *orc_model_block_table(int model, int *row_stride);
int orc_model_row_len(int model, int seq);

double orc_e4m3_decode(uint8_t code);
uint8_t orc_e4m3_encode(float y);   /* nearest value, ties to even code, saturating at 448 */
int orc_num_threads(void);
void orc_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
