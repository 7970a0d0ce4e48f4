// Internal declarations shared by the host API and the HIP kernels of libprismkv.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// built with hidden visibility: only what the public header declares is exported
#pragma GCC visibility push(default)
#include "../../include/prism_kv.h"
#include "../../include/prism_kv_tuning.h"
#pragma GCC visibility pop

#define PKV_MAX_POOLS 8
#define PKV_MAX_MODELS 64
#define PKV_FP8_HEADER 128   // bytes in front of an e4m3 block: fp32 sK[Hkv], fp32 sV[Hkv]
#define PKV_MAX_BATCH_OPS 4096   // entries of one reserve call (the growth rounds of a whole admission)
#define PKV_MAX_ROW_BLOCKS (1 << 20)   // blocks a row can hold at most (the reserve kernel packs a row position into 20 bits)
#define PKV_MAX_SEQS 4096
#define PKV_BOOK_THREADS 1024
// The file-scope scratch array of decode_attention_static: arrival counters, then split-K partials.
#define PKV_STATIC_COUNTERS 32768
#define PKV_STATIC_SCRATCH_BYTES ((size_t)20 << 20)

// Unsigned division by an invariant divisor with one multiply-high and two shifts
// (Granlund & Montgomery, "Division by invariant integers using multiplication").
// Exact for every 32-bit numerator.
struct FastDiv {
    uint32_t d, mul, sh1, sh2;
};

static inline FastDiv fastdiv_make(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;                   // l = ceil(log2 d)
    f.mul = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l < 1 ? 0 : l - 1;
    return f;
}

__host__ __device__ static inline uint32_t fastdiv_div(uint32_t n, const FastDiv &f) {
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t t = __umulhi(n, f.mul);
#else
    uint32_t t = (uint32_t)(((uint64_t)n * f.mul) >> 32);
#endif
    return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// Result slot in pinned host memory, written by the bookkeeping kernels.
struct BookResult {
    int64_t value;     // count or negative PKV_E_* code
    int64_t aux0, aux1;
};

// Device-resident pool state.
struct PoolDev {
    int32_t *owner;        // [n_frames] model id or -1
    uint32_t *free_stack;  // [n_frames], [0] bottom .. [n_free-1] top
    int32_t *pos;          // [n_frames] position of the frame in its owner's list
    int64_t *n_free;       // [1]
    int64_t n_frames;
};

// Device-resident per-model bookkeeping state.
struct ModelDev {
    uint32_t *frames;      // [n_frames] acquisition order
    uint32_t *bits;        // [n_frames][wpf] slot bits of the frame at that position
    uint8_t *mark;         // [n_frames] scratch for deflate
    int32_t *rows;         // [max_seqs][max_blocks] block ids
    int32_t *row_len;      // [max_seqs]
    int64_t *counters;     // [0] owned frames, [1] free slots
    int32_t model_id;
    int32_t slots, wpf;    // slots per frame, 32-bit words per frame in `bits`
    int32_t max_seqs, max_blocks, page_tokens;
};

// What one attention work-group needs to know about its model.
struct AttnDesc {
    const uint8_t *pool_base;
    const uint16_t *q;          // bf16 [B][Hq][D]
    const int32_t *table;       // [B][row_stride]
    const int32_t *ctx_lens;    // [B]
    const int32_t *row_len;     // library table: [max_seqs] blocks reserved per row; NULL for a caller's table
    const int4 *vmap;           // prefill launches: [groups] {sequence, first q/out row, chunk tokens after the
                                // group, tokens in the group}; chunk append: [units] {first new row of the
                                // sequence, its new tokens, sequence, which of the pages the chunk touches}
    float *out;                 // [B][Hq][D]
    float *ws;                  // split-K partials: two per work item (uncached memory)
    uint32_t *cnt;              // [B][Hkv] arrival counters of the split-K merge, zero between launches
    uint32_t *err;              // device error flags
    const void *safe;           // 16 KiB of zeros owned by the library: stands in for blocks that must not be read
    uint64_t frame_bytes, block_bytes;
    FastDiv slots_div;
    uint32_t max_block_id;      // n_frames * slots
    int32_t batch, row_stride;
    int32_t Hq, Hkv, g, D, dtype;
    int32_t cols;               // MFMA columns in use per kv head: (query tokens per row) * g, at most 16
    int32_t item_begin;         // first work item of this model in a grouped launch
    int32_t n_items;            // work items (waves) of this model
    int32_t min_share;          // smallest share of pages a wave may get
    int32_t weighted;           // items come in whole blocks of eight aligned with the XCDs
    int32_t seg_cost;           // what a segment costs besides its pages, in pages (for the split only)
    float scale_log2;           // log2(e) / sqrt(D)
};

#define PKV_MAX_GROUP 16
#define PKV_PREFILL_TILES 8     // tiles of query tokens per prefill work-group (4 waves x 2)

// How a launch cuts each block of eight consecutive shares among the eight XCDs.
struct AttnTune {
    uint32_t cum[9];            // cumulative weights in 1/65536: cum[0] = 0 <= ... <= cum[8] = 65536
    uint64_t *stat;             // NULL, or [8][2]: per XCD the sum of its waves' streaming times
                                // (100 MHz ticks) and their number; set in tuning launches only
};

struct AttnGroup {
    AttnDesc m[PKV_MAX_GROUP];
    AttnTune tune;
    int32_t n;
};

// ---- launch wrappers implemented in the .hip files ----------------------------
hipError_t pkv_launch_pool_init(const PoolDev &p, const uint32_t *perm_dev, hipStream_t s);
// Bookkeeping kernels: the result goes to *res (pinned host memory); a refused call also sets bit 2 of *err.
hipError_t pkv_launch_resize(const PoolDev &p, const ModelDev &m, int64_t target, BookResult *res, uint32_t *err, hipStream_t s);
// ops: pinned host memory, n sequence ids, n context lengths, then per entry the largest want (blocks) among
// the earlier entries of its sequence in the list (n <= PKV_MAX_BATCH_OPS)
hipError_t pkv_launch_reserve(const PoolDev &p, const ModelDev &m, int n, const int32_t *ops, BookResult *res, uint32_t *err,
                              hipStream_t s);
// ops: pinned host memory, n sequence ids (n <= PKV_MAX_SEQS)
hipError_t pkv_launch_release(const PoolDev &p, const ModelDev &m, int n, const int32_t *ops, BookResult *res, uint32_t *err,
                              hipStream_t s);

hipError_t pkv_launch_kv_write(const AttnDesc &d, int seq, int tok_begin, int n_tok, const void *k, const void *v,
                               const float *ks, const float *vs, int page_tokens, hipStream_t s);
hipError_t pkv_launch_kv_read(const AttnDesc &d, int seq, int tok_begin, int n_tok, void *k, void *v, float *ks, float *vs,
                              hipStream_t s);
// d.batch sequences, d.ctx_lens / d.row_len / d.table as for attention
hipError_t pkv_launch_kv_append(const AttnDesc &d, const void *k_new, const void *v_new, hipStream_t s);
// ev: NULL or two events recorded before and after the attention kernel
hipError_t pkv_launch_attention(const AttnGroup &grp, bool deep, hipStream_t s, hipEvent_t *ev);
// the entry point that allocates nothing: the current device's copy of the library's scratch array
hipError_t pkv_static_scratch(void **ptr);
hipError_t pkv_launch_attention_static(const AttnGroup &grp, uint32_t *cnt, size_t n_cnt, hipStream_t s);
// chunked prefill: d.vmap lists n_groups groups of up to PKV_PREFILL_TILES * (d.cols / d.g) query tokens
hipError_t pkv_launch_prefill(const AttnDesc &d, int n_groups, bool any_split, hipStream_t s);
hipError_t pkv_launch_stream_read(const void *src, size_t bytes, size_t granule_bytes, uint32_t *sink, hipStream_t s);
