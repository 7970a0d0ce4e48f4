// Page-pool / balloon bookkeeping kernels (gfx950).
//
// All state (free stack, frame ownership, per-model frame lists, slot bitmaps,
// block tables) lives in HBM and is changed only here.  The operations follow the
// balloon driver's contract in the paper (Sec. 4.2): D1 — a model's share grows and
// shrinks, memory only changes hands; D2 — token blocks fill slots of the model's
// own pages; D3 — partially filled pages are used first.  Results must be identical
// from run to run and equal to a sequential execution, so every ordering decision
// is taken with prefix sums inside ONE work-group of 1024 lanes; no atomics decide
// an order.  The data moved per call is a few KB, the cost is launch latency.
#include "pkv_internal.h"

namespace {

constexpr int NT = PKV_BOOK_THREADS;
constexpr int NW = NT / 64;

// Work-group barrier for exchanges through LDS only: it waits for this wave's LDS traffic, not for its
// global stores to be acknowledged (__syncthreads does, and a store's round trip costs about as much as
// everything else such a kernel does between two barriers).
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Exclusive prefix sum of one int per lane over the work-group; `total` is uniform.
__device__ inline int block_excl_scan(int v, int &total, int *s_wave) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    __syncthreads();                 // protect s_wave from the previous call's readers
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    int before = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        int x = s_wave[w];
        if (w < wave) before += x;
        sum += x;
    }
    total = sum;
    return before + inc - v;
}

__global__ void k_pool_init(PoolDev p, const uint32_t *perm) {
    const int64_t n = p.n_frames;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        p.owner[i] = -1;
        p.pos[i] = -1;
        // pops take from the top (the end): frame perm[0] (or 0) must be last
        p.free_stack[n - 1 - i] = perm ? perm[i] : (uint32_t)i;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *p.n_free = n;
}

// A call's result goes to its slot in pinned host memory; a refused call also raises the sticky
// device flag (bit 2), so that a caller who only enqueues learns of it without reading every slot.
__device__ inline void book_finish(BookResult *res, uint32_t *err, int64_t value) {
    if (value < 0 && err) atomicOr(err, 4u);
    __threadfence_system();
    res->value = value;
}

// inflate: pop `need` frames, append them to the model's list, all or nothing.
__device__ inline void inflate_body(const PoolDev &p, const ModelDev &m, int64_t target, BookResult *res, uint32_t *err) {
    const int64_t owned = m.counters[0];
    const int64_t n_free = *p.n_free;
    const int64_t need = target - owned;
    if (need <= 0) {
        if (threadIdx.x == 0) book_finish(res, err, owned);
        return;
    }
    if (need > n_free) {
        if (threadIdx.x == 0) book_finish(res, err, PKV_E_NOMEM);
        return;
    }
    for (int64_t k = threadIdx.x; k < need; k += NT) {
        const uint32_t f = p.free_stack[n_free - 1 - k];
        const int64_t at = owned + k;
        p.owner[f] = m.model_id;
        p.pos[f] = (int32_t)at;
        m.frames[at] = f;
        for (int w = 0; w < m.wpf; ++w) m.bits[at * m.wpf + w] = 0u;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        *p.n_free = n_free - need;
        m.counters[0] = target;
        m.counters[1] += need * m.slots;
        res->aux0 = need;
        book_finish(res, err, target);
    }
}

// deflate: hand back empty frames, newest first, until `target` is met (clamp at
// frames that still hold blocks); then close the gaps in the frame list and bitmap
// keeping the order of what stays.
__device__ inline void deflate_body(const PoolDev &p, const ModelDev &m, int64_t target, BookResult *res, uint32_t *err, int *s_wave) {
    const int tid = threadIdx.x;
    const int64_t owned = m.counters[0];
    const int64_t n_free = *p.n_free;
    const int64_t want = owned - target;
    if (want <= 0) {
        if (tid == 0) book_finish(res, err, owned);
        return;
    }
    const int wpf = m.wpf;
    int64_t reclaimed = 0, lo = owned;
    for (int64_t base = owned - 1; base >= 0 && reclaimed < want; base -= NT) {
        const int64_t i = base - tid;
        int empty = 0;
        if (i >= 0) {
            empty = 1;
            for (int w = 0; w < wpf; ++w)
                if (m.bits[i * wpf + w]) empty = 0;
        }
        int total;
        const int excl = block_excl_scan(empty, total, s_wave);   // rank in newest-first order
        const bool take = empty && (reclaimed + excl < want);
        if (i >= 0) m.mark[i] = take ? 1 : 0;
        if (take) {
            const uint32_t f = m.frames[i];
            p.free_stack[n_free + reclaimed + excl] = f;           // pushed in scan order
            p.owner[f] = -1;
            p.pos[f] = -1;
        }
        reclaimed += (total < want - reclaimed) ? total : (want - reclaimed);
        lo = (base - (NT - 1) > 0) ? base - (NT - 1) : 0;
    }
    __syncthreads();
    // compaction of positions [lo, owned): column by column, read - barrier - write.
    // A kept entry only moves down, onto a slot whose old content was read in this
    // or an earlier round.
    int64_t w_at = lo;
    for (int64_t base = lo; base < owned; base += NT) {
        const int64_t i = base + tid;
        const int keep = (i < owned) && !m.mark[i];
        int total;
        const int excl = block_excl_scan(keep, total, s_wave);
        const int64_t to = w_at + excl;
        uint32_t f = 0;
        if (keep) f = m.frames[i];
        __syncthreads();
        if (keep) {
            m.frames[to] = f;
            p.pos[f] = (int32_t)to;
        }
        for (int w = 0; w < wpf; ++w) {
            uint32_t b = 0;
            if (keep) b = m.bits[i * wpf + w];
            __syncthreads();
            if (keep) m.bits[to * wpf + w] = b;
        }
        w_at += total;
        __syncthreads();
    }
    if (tid == 0) {
        *p.n_free = n_free + reclaimed;
        m.counters[0] = owned - reclaimed;
        m.counters[1] -= reclaimed * m.slots;
        res->aux0 = reclaimed;
        book_finish(res, err, owned - reclaimed);
    }
}

// balloon_resize: the direction is decided here, from the device's own count of owned frames, so
// that a caller can enqueue the call without knowing how earlier enqueued calls ended.
__global__ __launch_bounds__(NT) void k_resize(PoolDev p, ModelDev m, int64_t target, BookResult *res, uint32_t *err) {
    __shared__ int s_wave[NW];
    const int64_t owned = m.counters[0];          // uniform: every lane takes the same branch
    if (target > owned) inflate_body(p, m, target, res, err);
    else if (target < owned) deflate_body(p, m, target, res, err, s_wave);
    else if (threadIdx.x == 0) book_finish(res, err, owned);
}

// reserve (batched): rows grow to ceil(ctx / T) blocks; the new blocks of the whole
// batch take the lowest free slots in frame-list order, entry by entry — the same
// state a sequential loop of single reserves leaves.  A sequence may appear several
// times (the growth rounds of an admission in one call): entry i then needs what its
// row lacks after the earlier entries, i.e. its want minus the largest want among the
// earlier entries of the same sequence (and the row's length before the call).
// ops: host (pinned) memory, n sequence ids, then n context lengths, then for each entry the largest want
// (in blocks) among the earlier entries of its sequence in this list, 0 if there is none.
__global__ __launch_bounds__(NT) void k_reserve(PoolDev p, ModelDev m, int n, const int32_t *ops, BookResult *res, uint32_t *err) {
    __shared__ int s_wave[NW];
    __shared__ int s_cur[PKV_MAX_SEQS];             // row lengths: as the call finds them, then with its wants
    __shared__ int s_start[PKV_MAX_BATCH_OPS + 1];  // first rank of entry i
    __shared__ uint32_t s_ent[PKV_MAX_BATCH_OPS];   // entry i: sequence << 20 | row length before the entry
    __shared__ uint32_t s_free[NT], s_fid[NT];      // placement: free bits of frame j's current word, its frame id
    __shared__ int s_rank[NT];                      // placement: rank of the first free slot of that word
    __shared__ int s_fail;
    const int tid = threadIdx.x;
    // Everything the kernel will read is asked for here, before the first answer is needed: the list
    // (host memory, the longest trip), the rows' lengths, the counters and the lane's own frame of the
    // first pass of the placement.  The call then costs one such trip instead of five in a row.
    constexpr int CHUNKS = PKV_MAX_BATCH_OPS / NT, PRE_WORDS = 4;
    int o_seq[CHUNKS], o_ctx[CHUNKS], o_ear[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        const int i = c * NT + tid;
        o_seq[c] = i < n ? ops[i] : 0;
        o_ctx[c] = i < n ? ops[n + i] : 0;
        o_ear[c] = i < n ? ops[2 * n + i] : 0;
    }
    const int64_t owned = m.counters[0], spare = m.counters[1];
    const int wpf = m.wpf, slots = m.slots;
    uint32_t pre_bits[PRE_WORDS];
    // (list positions the model does not own yet are read too, and never looked at: the address then does
    // not wait for the count of owned frames to arrive)
#pragma unroll
    for (int w = 0; w < PRE_WORDS; ++w) pre_bits[w] = (tid < p.n_frames && w < wpf) ? m.bits[(int64_t)tid * wpf + w] : 0u;
    const uint32_t pre_frame = tid < p.n_frames ? m.frames[tid] : 0u;
    for (int s = tid; s < m.max_seqs; s += NT) s_cur[s] = m.row_len[s];
    if (tid == 0) s_fail = 0x7fffffff;
    __syncthreads();
    const int T = m.page_tokens;
    // Row length before an entry = the larger of the row's length when the call began and the largest want
    // among the earlier entries of its sequence.  The second is a property of the list alone and comes
    // with it; the first is read here, for every entry, before any entry's want reaches s_cur.
    int e_seq[CHUNKS], e_want[CHUNKS], e_prev[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        const int i = c * NT + tid;
        e_seq[c] = -1;
        e_want[c] = e_prev[c] = 0;
        if (i < n) {
            const int s_ = o_seq[c], cl = o_ctx[c];
            if (s_ < 0 || s_ >= m.max_seqs || cl < 0) {
                atomicMin(&s_fail, i * 2);                       // the first refused entry decides the code
            } else {
                const int64_t w = ((int64_t)cl + T - 1) / T;
                if (w > m.max_blocks) atomicMin(&s_fail, i * 2 + 1);
                else {
                    e_seq[c] = s_;
                    e_want[c] = (int)w;
                    const int before = s_cur[s_];
                    e_prev[c] = before > o_ear[c] ? before : o_ear[c];
                }
            }
        }
    }
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        const int c0 = c * NT, i = c0 + tid;
        if (c0 >= n) break;                                      // uniform
        const int seq = e_seq[c], want = e_want[c], prev = e_prev[c];
        if (seq >= 0) atomicMax(&s_cur[seq], want);              // the row's length after the call
        const int need = (seq >= 0 && want > prev) ? want - prev : 0;
        int chunk_total;
        const int excl = block_excl_scan(need, chunk_total, s_wave);
        if (i < n) {
            s_start[i] = total + excl;
            s_ent[i] = ((uint32_t)(seq >= 0 ? seq : 0) << 20) | (uint32_t)prev;
        }
        total += chunk_total;
    }
    if (tid == 0) s_start[n] = total;
    __syncthreads();
    int status = 0;
    if (s_fail != 0x7fffffff) status = (s_fail & 1) ? PKV_E_RANGE : PKV_E_ARG;
    else if ((int64_t)total > spare) status = PKV_E_BALLOON;
    if (status != 0 || total == 0) {
        if (tid == 0) book_finish(res, err, status);
        return;
    }
    // Placement.  Free slots are ranked in frame-list order, ascending slot inside a frame; rank r goes to
    // the entry e with s_start[e] <= r < s_start[e + 1].  A lane per frame counts the frame's free slots (a
    // prefix sum gives the rank of its first one) and publishes one 32-slot word at a time; then a lane per
    // (frame, slot) of that word takes over: a free slot knows its rank from the bits below it, finds its
    // entry by binary search and writes the row.  The frame's lane sets the bits that were taken.
    int running = 0;
    for (int64_t base = 0; base < owned && running < total; base += NT) {
        const int64_t i = base + tid;
        const bool pre = base == 0 && wpf <= PRE_WORDS;      // this pass's words are already here
        auto word_of = [&](int w) {
            uint32_t word = 0u;
            if (pre) {
#pragma unroll
                for (int k = 0; k < PRE_WORDS; ++k)
                    if (k == w) word = pre_bits[k];
            } else {
                word = m.bits[i * wpf + w];
            }
            return word;
        };
        auto valid_of = [&](int w) {
            const int nb = slots - 32 * w;
            return nb >= 32 ? 0xffffffffu : ((1u << nb) - 1u);
        };
        int zeros = 0;
        if (i < owned)
            for (int w = 0; w < wpf; ++w) zeros += __popc(~word_of(w) & valid_of(w));
        int chunk_total;
        int rank0 = running + block_excl_scan(zeros, chunk_total, s_wave);    // rank of this frame's first free slot
        const uint32_t f = i < owned ? (base == 0 ? pre_frame : m.frames[i]) : 0u;
        const int nf = (int)(owned - base < NT ? owned - base : NT);
        for (int w = 0; w < wpf; ++w) {
            const bool mine = i < owned && zeros && rank0 < total;
            const uint32_t word = mine ? word_of(w) : 0u;
            const uint32_t freeb = mine ? ~word & valid_of(w) : 0u;
            s_free[tid] = freeb;
            s_rank[tid] = rank0;
            s_fid[tid] = f;
            lds_barrier();
            for (int idx = tid; idx < nf * 32; idx += NT) {
                const int j = idx >> 5, bit = idx & 31;
                const uint32_t fr = s_free[j];
                if (!((fr >> bit) & 1u)) continue;
                const int r = s_rank[j] + __popc(fr & ((1u << bit) - 1u));
                if (r >= total) continue;
                // last entry with s_start <= r: three pivots a step (their reads travel together), then halves
                int lo = 0, hi = n;
                while (hi - lo > 3) {
                    const int q = (hi - lo) >> 2;
                    const int m1 = lo + q, m2 = m1 + q, m3 = m2 + q;
                    const int a1 = s_start[m1], a2 = s_start[m2], a3 = s_start[m3];
                    if (a3 <= r) lo = m3;
                    else if (a2 <= r) { lo = m2; hi = m3; }
                    else if (a1 <= r) { lo = m1; hi = m2; }
                    else hi = m1;
                }
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (s_start[mid] <= r) lo = mid; else hi = mid;
                }
                const uint32_t ent = s_ent[lo];
                m.rows[(int64_t)(ent >> 20) * m.max_blocks + (ent & 0xfffffu) + (r - s_start[lo])] =
                    (int32_t)(s_fid[j] * (uint32_t)slots + (uint32_t)(32 * w + bit));
            }
            lds_barrier();
            if (freeb) {
                const int c = __popc(freeb);
                int take = total - rank0;
                take = take > c ? c : take;
                uint32_t mask = freeb;                   // the lowest `take` free bits
                if (take < c) {
                    mask = 0u;
                    uint32_t rest = freeb;
                    for (int k = 0; k < take; ++k) {
                        mask |= rest & (0u - rest);
                        rest &= rest - 1u;
                    }
                }
                m.bits[i * wpf + w] = word | mask;
                rank0 += c;
            }
        }
        running += chunk_total;
    }
    __syncthreads();
    for (int s = tid; s < m.max_seqs; s += NT) m.row_len[s] = s_cur[s];
    if (tid == 0) {
        m.counters[1] = spare - total;
        book_finish(res, err, total);
    }
}

constexpr int RELEASE_WIN = 6144;      // words of a model's slot bitmap that k_release collects in LDS at a time

// release (batched): clear the slot bits of every block of the listed rows; the same state as single
// releases in order (a sequence listed twice is empty the second time).
// ops: host (pinned) memory, n sequence ids, checked by the host.
__global__ __launch_bounds__(NT) void k_release(PoolDev p, ModelDev m, int n, const int32_t *ops, BookResult *res, uint32_t *err) {
    __shared__ int s_wave[NW];
    __shared__ int s_start[PKV_MAX_SEQS + 1];
    __shared__ int s_seq[PKV_MAX_SEQS];
    __shared__ uint32_t s_win[RELEASE_WIN];
    const int tid = threadIdx.x;
    for (int i = tid; i < n; i += NT) {
        const int s_ = ops[i];
        s_seq[i] = (s_ >= 0 && s_ < m.max_seqs) ? s_ : -1;
    }
    __syncthreads();
    int total = 0;
    for (int c0 = 0; c0 < n; c0 += NT) {
        const int i = c0 + tid;
        int len = 0;
        if (i < n && s_seq[i] >= 0) {
            len = m.row_len[s_seq[i]];
            for (int j = 0; j < i && len > 0; ++j)       // listed before: already empty
                if (s_seq[j] == s_seq[i]) len = 0;
        }
        int chunk_total;
        const int excl = block_excl_scan(len, chunk_total, s_wave);
        if (i < n) s_start[i] = total + excl;
        total += chunk_total;
    }
    if (tid == 0) s_start[n] = total;
    __syncthreads();
    // Every block costs two dependent reads (its id in the row, then the list position of its frame)
    // before its bit can be cleared; a lane takes RELEASE_BATCH blocks at a time and issues each kind of
    // read for all of them before it needs the first answer, so a pass costs two memory round trips.
    // The bits to clear are collected in LDS, a window of WIN words of the model's slot bitmap at a
    // time (one window covers the bitmap of all but very large models), and each word that lost bits is
    // then rewritten once by one lane: thirty atomics on the same word in memory cost more than the
    // rest of the kernel.
    constexpr int RELEASE_BATCH = 8;
    const int64_t words_total = m.counters[0] * m.wpf;
    for (int64_t win0 = 0; win0 < words_total && total > 0; win0 += RELEASE_WIN) {
        for (int i = tid; i < RELEASE_WIN; i += NT) s_win[i] = 0u;
        lds_barrier();
        for (int x0 = 0; x0 < total; x0 += NT * RELEASE_BATCH) {
            uint32_t id[RELEASE_BATCH];
            int64_t at[RELEASE_BATCH];
#pragma unroll
            for (int u = 0; u < RELEASE_BATCH; ++u) {
                const int x = x0 + u * NT + tid;
                id[u] = 0xffffffffu;
                if (x < total) {
                    int lo = 0, hi = n;                      // last entry with s_start <= x
                    while (hi - lo > 1) {
                        const int mid = (lo + hi) >> 1;
                        if (s_start[mid] <= x) lo = mid; else hi = mid;
                    }
                    id[u] = (uint32_t)m.rows[(int64_t)s_seq[lo] * m.max_blocks + (x - s_start[lo])];
                }
            }
#pragma unroll
            for (int u = 0; u < RELEASE_BATCH; ++u)
                at[u] = id[u] != 0xffffffffu ? p.pos[id[u] / (uint32_t)m.slots] : 0;
#pragma unroll
            for (int u = 0; u < RELEASE_BATCH; ++u)
                if (id[u] != 0xffffffffu) {
                    const uint32_t sl = id[u] % (uint32_t)m.slots;
                    const int64_t word = at[u] * m.wpf + (sl >> 5) - win0;
                    if (word >= 0 && word < RELEASE_WIN) atomicOr(&s_win[word], 1u << (sl & 31));
                }
        }
        lds_barrier();
        for (int i = tid; i < RELEASE_WIN && win0 + i < words_total; i += NT) {
            const uint32_t gone = s_win[i];
            if (gone) m.bits[win0 + i] &= ~gone;
        }
        lds_barrier();
    }
    __syncthreads();
    for (int i = tid; i < n; i += NT)
        if (s_seq[i] >= 0) m.row_len[s_seq[i]] = 0;
    if (tid == 0) {
        m.counters[1] += total;
        book_finish(res, err, total);
    }
}

}  // namespace

hipError_t pkv_launch_pool_init(const PoolDev &p, const uint32_t *perm_dev, hipStream_t s) {
    int blocks = (int)((p.n_frames + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_pool_init, dim3(blocks), dim3(256), 0, s, p, perm_dev);
    return hipGetLastError();
}
hipError_t pkv_launch_resize(const PoolDev &p, const ModelDev &m, int64_t target, BookResult *res, uint32_t *err, hipStream_t s) {
    hipLaunchKernelGGL(k_resize, dim3(1), dim3(NT), 0, s, p, m, target, res, err);
    return hipGetLastError();
}
hipError_t pkv_launch_reserve(const PoolDev &p, const ModelDev &m, int n, const int32_t *ops, BookResult *res, uint32_t *err,
                              hipStream_t s) {
    hipLaunchKernelGGL(k_reserve, dim3(1), dim3(NT), 0, s, p, m, n, ops, res, err);
    return hipGetLastError();
}
hipError_t pkv_launch_release(const PoolDev &p, const ModelDev &m, int n, const int32_t *ops, BookResult *res, uint32_t *err,
                              hipStream_t s) {
    hipLaunchKernelGGL(k_release, dim3(1), dim3(NT), 0, s, p, m, n, ops, res, err);
    return hipGetLastError();
}
