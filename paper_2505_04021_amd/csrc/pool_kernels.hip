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

// inflate: pop `need` frames, append them to the model's list, all or nothing.
__global__ __launch_bounds__(NT) void k_inflate(PoolDev p, ModelDev m, int64_t target, BookResult *res) {
    const int64_t owned = m.counters[0];
    const int64_t n_free = *p.n_free;
    const int64_t need = target - owned;
    if (need <= 0) {
        if (threadIdx.x == 0) res->value = owned;
        return;
    }
    if (need > n_free) {
        if (threadIdx.x == 0) res->value = PKV_E_NOMEM;
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
        __threadfence_system();
        res->value = target;
    }
}

// deflate: hand back empty frames, newest first, until `target` is met (clamp at
// frames that still hold blocks); then close the gaps in the frame list and bitmap
// keeping the order of what stays.
__global__ __launch_bounds__(NT) void k_deflate(PoolDev p, ModelDev m, int64_t target, BookResult *res) {
    __shared__ int s_wave[NW];
    const int tid = threadIdx.x;
    const int64_t owned = m.counters[0];
    const int64_t n_free = *p.n_free;
    const int64_t want = owned - target;
    if (want <= 0) {
        if (tid == 0) res->value = owned;
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
        __threadfence_system();
        res->value = owned - reclaimed;
    }
}

// reserve (batched): rows grow to ceil(ctx / T) blocks; the new blocks of the whole
// batch take the lowest free slots in frame-list order, entry by entry — the same
// state a sequential loop of single reserves leaves.
__global__ __launch_bounds__(NT) void k_reserve(PoolDev p, ModelDev m, int n, const int32_t *ops, BookResult *res) {
    __shared__ int s_wave[NW];
    __shared__ int s_cur[4096];                     // row length while walking the batch
    __shared__ int s_start[PKV_MAX_BATCH_OPS + 1];  // first rank of entry i
    __shared__ int s_base[PKV_MAX_BATCH_OPS];       // row length before entry i
    __shared__ int s_seq[PKV_MAX_BATCH_OPS];
    __shared__ int s_ctx[PKV_MAX_BATCH_OPS];
    __shared__ int s_status, s_total;
    const int tid = threadIdx.x;
    for (int s = tid; s < m.max_seqs; s += NT) s_cur[s] = m.row_len[s];
    for (int i = tid; i < n; i += NT) {          // ops sits in host memory: fetch it once, in parallel
        s_seq[i] = ops[i];
        s_ctx[i] = ops[n + i];
    }
    __syncthreads();
    if (tid == 0) {
        int total = 0, status = 0;
        const int T = m.page_tokens;
        for (int i = 0; i < n; ++i) {
            const int s = s_seq[i], c = s_ctx[i];
            if (s < 0 || s >= m.max_seqs || c < 0) { status = PKV_E_ARG; break; }
            const int want = (int)(((int64_t)c + T - 1) / T);
            if (want > m.max_blocks) { status = PKV_E_RANGE; break; }
            const int need = want > s_cur[s] ? want - s_cur[s] : 0;
            s_start[i] = total;
            s_base[i] = s_cur[s];
            s_cur[s] += need;
            total += need;
        }
        s_start[n] = total;
        if (status == 0 && (int64_t)total > m.counters[1]) status = PKV_E_BALLOON;
        s_status = status;
        s_total = total;
    }
    __syncthreads();
    const int status = s_status, total = s_total;
    if (status != 0 || total == 0) {
        if (tid == 0) res->value = status;
        return;
    }
    const int64_t owned = m.counters[0];
    const int wpf = m.wpf, slots = m.slots;
    int running = 0;
    for (int64_t base = 0; base < owned && running < total; base += NT) {
        const int64_t i = base + tid;
        int zeros = 0;
        if (i < owned) {
            for (int w = 0; w < wpf; ++w) {
                const int nb = slots - 32 * w;
                const uint32_t valid = nb >= 32 ? 0xffffffffu : ((1u << nb) - 1u);
                zeros += __popc(~m.bits[i * wpf + w] & valid);
            }
        }
        int chunk_total;
        int r = running + block_excl_scan(zeros, chunk_total, s_wave);
        if (zeros && r < total) {
            const uint32_t f = m.frames[i];
            int lo = 0, hi = n;                      // last entry with s_start <= r
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_start[mid] <= r) lo = mid; else hi = mid;
            }
            for (int w = 0; w < wpf && r < total; ++w) {
                const int nb = slots - 32 * w;
                const uint32_t valid = nb >= 32 ? 0xffffffffu : ((1u << nb) - 1u);
                uint32_t word = m.bits[i * wpf + w];
                uint32_t freeb = ~word & valid;
                while (freeb && r < total) {
                    const int b = __ffs(freeb) - 1;
                    freeb &= freeb - 1;
                    while (s_start[lo + 1] <= r) ++lo;   // ranks rise by one: walk forward
                    m.rows[(int64_t)s_seq[lo] * m.max_blocks + s_base[lo] + (r - s_start[lo])] =
                        (int32_t)(f * (uint32_t)slots + (uint32_t)(32 * w + b));
                    word |= 1u << b;
                    ++r;
                }
                m.bits[i * wpf + w] = word;
            }
        }
        running += chunk_total;
    }
    __syncthreads();
    for (int s = tid; s < m.max_seqs; s += NT) m.row_len[s] = s_cur[s];
    if (tid == 0) {
        m.counters[1] -= total;
        __threadfence_system();
        res->value = total;
    }
}

// release: clear the slot bits of every block of the row.
__global__ __launch_bounds__(NT) void k_release(PoolDev p, ModelDev m, int seq, BookResult *res) {
    const int n = m.row_len[seq];
    for (int b = threadIdx.x; b < n; b += NT) {
        const uint32_t id = (uint32_t)m.rows[(int64_t)seq * m.max_blocks + b];
        const uint32_t f = id / (uint32_t)m.slots, s = id % (uint32_t)m.slots;
        const int64_t at = p.pos[f];
        atomicAnd(&m.bits[at * m.wpf + (s >> 5)], ~(1u << (s & 31)));
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        m.row_len[seq] = 0;
        m.counters[1] += n;
        __threadfence_system();
        res->value = n;
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
hipError_t pkv_launch_inflate(const PoolDev &p, const ModelDev &m, int64_t target, BookResult *res, hipStream_t s) {
    hipLaunchKernelGGL(k_inflate, dim3(1), dim3(NT), 0, s, p, m, target, res);
    return hipGetLastError();
}
hipError_t pkv_launch_deflate(const PoolDev &p, const ModelDev &m, int64_t target, BookResult *res, hipStream_t s) {
    hipLaunchKernelGGL(k_deflate, dim3(1), dim3(NT), 0, s, p, m, target, res);
    return hipGetLastError();
}
hipError_t pkv_launch_reserve(const PoolDev &p, const ModelDev &m, int n, const int32_t *ops, BookResult *res, hipStream_t s) {
    hipLaunchKernelGGL(k_reserve, dim3(1), dim3(NT), 0, s, p, m, n, ops, res);
    return hipGetLastError();
}
hipError_t pkv_launch_release(const PoolDev &p, const ModelDev &m, int seq, BookResult *res, hipStream_t s) {
    hipLaunchKernelGGL(k_release, dim3(1), dim3(NT), 0, s, p, m, seq, res);
    return hipGetLastError();
}
