// Host side of libprismkv: the C-ABI of include/prism_kv.h.
//
// Handles argument checks, device allocations and kernel launches.  It never
// computes bookkeeping or attention results itself: the page-pool state lives in
// HBM and changes only through the kernels in pool_kernels.hip; the host keeps just
// the shapes and a shadow of each row's length (a deterministic function of the
// successful calls) for argument validation.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

#include "pkv_internal.h"

static int tune_setup();      // buffers of the XCD weight tuning (defined with the tuning code)

namespace {

struct Pool {
    bool live = false;
    size_t bytes = 0, frame_bytes = 0;
    int T = 0;
    int64_t n_frames = 0;
    uint8_t *base = nullptr;
    bool own_base = false;
    PoolDev dev{};
    int64_t n_free = 0;                     // shadow of the device counter
    // elastic pools: `base` is a reserved address range; a frame is backed by memory while a model owns
    // it or while it waits, near the top of the free stack, in the pre-allocation buffer
    bool elastic = false;
    struct Elastic *el = nullptr;
};

// The memory side of an elastic pool (paper Sec. 4.2, D3: a pre-allocation thread keeps a buffer of pages
// ready, so that mapping cost stays off the critical path).  The free stack hands frames out from its
// top, so the buffer is simply "the top `target` frames of the free stack are backed by memory": an
// inflate of up to that many frames finds them ready and maps nothing; a deflate pushes its (mapped)
// frames on top and returns at once.  A worker thread restores the rule behind the caller's back: it maps
// frames that have risen into the top region and unmaps free frames that have sunk below it.  The host
// keeps a copy of the free stack for that (every change of the stack goes through balloon_resize, which
// on an elastic pool waits for its kernel and knows the frames that moved).
enum : uint8_t { F_UNMAPPED = 0, F_MAPPING, F_MAPPED, F_UNMAPPING };
struct Elastic {
    std::mutex mu;
    std::condition_variable work, done;     // work: something for the worker; done: a frame changed state / the worker is idle
    std::thread worker;
    bool stop = false, idle = true;
    uint64_t changes = 0, seen = 0;         // callers count every change of stack or target; the worker notes the count it has dealt with
    int device = 0;
    uint8_t *base = nullptr;
    size_t frame_bytes = 0;
    std::vector<uint32_t> stack;            // copy of the free stack, bottom .. top
    std::vector<uint8_t> state;             // per frame
    std::vector<hipMemGenericAllocationHandle_t> handle;    // per frame, valid unless F_UNMAPPED
    size_t target = 0;                      // frames of the buffer
    size_t low_water = 0;                   // every stack position below holds an unmapped frame
    int64_t mapped_frames = 0;              // frames not F_UNMAPPED
    int64_t mapped_free = 0;                // of those, frames no model owns
};

struct Model {
    bool live = false;
    int pool = -1;
    int Hq = 0, Hkv = 0, D = 0, dtype = 0, g = 0;
    int L = 1, layer = 0;                   // layers sharing the block table; the layer the KV calls address
    size_t layer_bytes = 0;                 // one layer's part of a block
    size_t block_bytes = 0;                 // all layers: L * layer_bytes
    int slots = 0;
    int batch = 0, row_stride = 0;          // model_set_batch
    int64_t owned = 0;                      // shadow of the device counter
    int64_t used_blocks = 0;
    std::vector<int32_t> row_len;           // shadow
    std::vector<int32_t> list_max;          // scratch of enqueue_reserve, all zero between calls
    // The shadows follow the calls as if each had succeeded in full.  After an enqueue-only bookkeeping
    // call nobody has looked at the outcome yet: the shadows are then estimates (good for sizing a
    // launch) until reconcile() has read the device's own counts back.
    bool stale = false;
    ModelDev dev{};
    float *ws = nullptr;                    // split-K partials
    size_t ws_floats = 0;
    uint32_t *cnt = nullptr;                // arrival counters, zero between launches
    size_t cnt_cap = 0;
    int4 *vmap = nullptr;                   // device: the rows (query tiles) of the last prefill launch
    size_t vmap_cap = 0;
    float *pf_ws = nullptr;                 // device: partial results of prefill groups whose context is split
    size_t pf_ws_floats = 0;
};

// Uncached device memory for split-K partials and arrival counters.  Blocks are
// recycled between models but never returned to the driver while the process lives.
struct UcBlock {
    void *p;
    size_t bytes;
    bool used;
};
std::vector<UcBlock> g_uc;

void *uc_alloc(size_t bytes) {
    int best = -1;
    for (size_t i = 0; i < g_uc.size(); ++i)
        if (!g_uc[i].used && g_uc[i].bytes >= bytes && (best < 0 || g_uc[i].bytes < g_uc[best].bytes)) best = (int)i;
    if (best < 0) {
        void *p = nullptr;
        if (hipExtMallocWithFlags(&p, bytes, hipDeviceMallocUncached) != hipSuccess) return nullptr;
        g_uc.push_back(UcBlock{p, bytes, false});
        best = (int)g_uc.size() - 1;
    }
    g_uc[best].used = true;
    return g_uc[best].p;
}

void uc_release(void *p) {
    for (auto &b : g_uc)
        if (b.p == p) b.used = false;
}

Pool g_pools[PKV_MAX_POOLS];
Model g_models[PKV_MAX_MODELS];
int g_last_pool = -1;
hipStream_t g_stream = nullptr;
// Bookkeeping calls run as kernels whose result lands in a slot of pinned host memory.  A call takes
// the next slot of a ring (its ticket); the synchronous forms wait for their slot, the enqueue-only
// forms hand the ticket to the caller.  A slot also carries the call's host-side operands (the list
// of a reserve / release batch), which its kernel reads straight from pinned memory.
constexpr int kTickets = 128;
constexpr int64_t kPending = INT64_MIN;
struct Ticket {
    long id = -1;
    hipStream_t stream = nullptr;
};
BookResult *g_res = nullptr;       // pinned host, [kTickets]
int32_t *g_ops = nullptr;          // pinned host, [kTickets][3 * PKV_MAX_BATCH_OPS]
Ticket g_tickets[kTickets];
long g_next_ticket = 0;
uint32_t *g_err = nullptr;         // device error flags
uint32_t g_host_flags = 0;         // the same flags, raised by the host (an enqueue-only call refused before any kernel ran)
void *g_safe = nullptr;            // 16 KiB of zeros: what kernels read instead of a block they must not touch
int g_items = 0, g_min_share = 0, g_seg_cost = -1;
int g_deep_mode = -1;                // which form of the attention kernel: -1 = by the launch, 0 = two waves per SIMD, 1 = one
bool g_deep_now = false;             // the form chosen for the launch being prepared
// How a block of eight shares is cut among the XCDs: weights (mean 1), and the state of a
// tuning run that derives them from when each XCD's waves finish.
float g_xcd_w[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
// The library tunes the weights itself, without ever waiting: while updates are still owed, a launch
// that fills the chip lets its waves add their streaming times to per-XCD sums on the device (running
// totals, never cleared); a copy of the totals travels to pinned host memory behind the launch, and a
// later launch that finds such a copy complete turns the difference to the previous copy into the
// next step of the weights.  What the XCDs differ by depends on the load (a launch that saturates the
// memory wants every second XCD some 7 % below the others, one whose waves are half bound by their own
// arithmetic wants equal shares), so after the updates a process starts with the weights keep
// following the launches, slowly: every kSlowTuneEvery-th launch that fills the chip is measured and
// moves them by a tenth of the way.
constexpr int kAutoTuneUpdates = 24;        // weight updates a process starts with (coarse ones first)
constexpr int kSlowTuneEvery = 8;
constexpr double kSlowTuneGain = 0.1;
constexpr int kTuneSlots = 4;
constexpr int kMinTuneItems = 256;          // smaller launches do not fill the chip: their times say little
uint64_t *g_xcd_stat = nullptr;             // device: [8][2] running sums of streaming time and wave counts
uint64_t *g_tune_host = nullptr;            // pinned: [kTuneSlots][16] copies of the totals
hipEvent_t g_tune_ev[kTuneSlots];
bool g_tune_busy[kTuneSlots];
long g_tune_version[kTuneSlots];            // which set of weights the launch behind the copy ran with
uint64_t g_tune_last[16];                   // the totals of the last copy looked at
long g_xcd_version = 0;                     // counts changes of the weights
int g_tune_left = kAutoTuneUpdates, g_tune_done = 0, g_tune_measured = 0;
bool g_tune_follow = true;                  // keep following the launches once the first updates are done
long g_tune_tick = 0;
constexpr int kMaxTuneMeasured = 4096;      // give up measuring if the updates never come (launches too alike in time)
constexpr float kXcdWeightMin = 0.75f, kXcdWeightMax = 1.25f;
double g_page_cost = -1.0;           // fixed cost of a page relative to 0.1 per KiB (< 0: the default of the kernel form)
int g_fail_map_after = -1;        // test hook: the (n+1)-th frame mapping from now fails as if memory had run out
int g_timing = 0;                 // 0 = off, n = bracket every n-th attention launch with events
long g_launches = 0;
std::vector<hipEvent_t> g_events;   // pairs: before and after the attention kernel
size_t g_events_used = 0;
constexpr size_t kMaxTimedLaunches = 8192;
thread_local char g_errbuf[256] = "";

int fail_hip(hipError_t e, const char *what) {
    snprintf(g_errbuf, sizeof g_errbuf, "%s: %s", what, hipGetErrorString(e));
    return PKV_E_DEVICE;
}
#define HIP_TRY(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) return fail_hip(e_, #call); \
    } while (0)

int lib_init() {
    if (g_res) return PKV_OK;
    HIP_TRY(hipHostMalloc((void **)&g_res, sizeof(BookResult) * kTickets, hipHostMallocDefault));
    for (int i = 0; i < kTickets; ++i) g_res[i].value = 0;
    HIP_TRY(hipHostMalloc((void **)&g_ops, sizeof(int32_t) * 3 * PKV_MAX_BATCH_OPS * kTickets, hipHostMallocDefault));
    HIP_TRY(hipMalloc((void **)&g_err, sizeof(uint32_t)));
    HIP_TRY(hipMemset(g_err, 0, sizeof(uint32_t)));
    HIP_TRY(hipMalloc(&g_safe, 16384));
    HIP_TRY(hipMemset(g_safe, 0, 16384));
    void *scratch_ptr = nullptr;          // resolve the current device's scratch array once, at set-up
    HIP_TRY(pkv_static_scratch(&scratch_ptr));
    return tune_setup();
}

Pool *get_pool(int id) { return (id >= 0 && id < PKV_MAX_POOLS && g_pools[id].live) ? &g_pools[id] : nullptr; }
Model *get_model(int id) { return (id >= 0 && id < PKV_MAX_MODELS && g_models[id].live) ? &g_models[id] : nullptr; }

// The next slot of the ring.  A slot whose previous call has not finished yet (its kernel still
// reads the slot's operands) is waited for first.
int take_ticket() {
    const long id = g_next_ticket++;
    const int slot = (int)(id % kTickets);
    if (g_tickets[slot].id >= 0 && g_res[slot].value == kPending) (void)hipStreamSynchronize(g_tickets[slot].stream);
    g_tickets[slot].id = id;
    g_tickets[slot].stream = g_stream;
    g_res[slot].value = kPending;
    g_res[slot].aux0 = g_res[slot].aux1 = 0;
    return slot;
}

int32_t *ticket_ops(int slot) { return g_ops + (size_t)slot * 3 * PKV_MAX_BATCH_OPS; }
int ticket_handle(int slot) { return (int)(g_tickets[slot].id & 0x7fffffff); }

// a call that was refused before anything was enqueued still gets a (finished) ticket
int finished_ticket(int64_t value) {
    const int slot = take_ticket();
    g_res[slot].value = value;
    return slot;
}

// Wait for a slot's kernel and return its result.  The kernel writes the slot when it ends, so the
// host watches the slot rather than the stream: work enqueued behind the call (a decode step) is
// not waited for.  The stream is asked now and then, so that a failed launch cannot hang the caller.
int64_t wait_ticket(int slot) {
    volatile int64_t *v = &g_res[slot].value;
    for (long spin = 0; *v == kPending; ++spin) {
        if ((spin & 1023) != 1023) continue;
        const hipError_t e = hipStreamQuery(g_tickets[slot].stream);
        if (e == hipErrorNotReady) continue;
        if (e != hipSuccess) return fail_hip(e, "bookkeeping call");
        break;                                        // the stream is idle: the kernel has ended
    }
    const int64_t r = *v;
    return r == kPending ? (int64_t)PKV_E_INTERNAL : r;
}

void free_model_dev(Model &m) {
    (void)hipFree(m.dev.frames); (void)hipFree(m.dev.bits); (void)hipFree(m.dev.mark); (void)hipFree(m.dev.rows);
    (void)hipFree(m.dev.row_len); (void)hipFree(m.dev.counters);
    uc_release(m.ws);
    uc_release(m.cnt);
    (void)hipFree(m.vmap);
    m.vmap = nullptr;
    m.vmap_cap = 0;
    (void)hipFree(m.pf_ws);
    m.pf_ws = nullptr;
    m.pf_ws_floats = 0;
    m.dev = ModelDev{};
    m.ws = nullptr;
    m.cnt = nullptr;
    m.ws_floats = m.cnt_cap = 0;
}

// Work items (waves) of an attention launch, and which form of the kernel runs them.
//
// The ordinary form has two waves per SIMD, and a launch of it gets what the chip holds at once (256
// CUs x 4 SIMDs x 2 = 2048 items): every wave starts at once and takes one equal share of the pages.
// More, smaller items were measured to be slower: an item that starts while the memory system is
// saturated pays ~10 us before its first page arrives.
//
// The second form has one wave per SIMD, and only as many waves as it takes to keep the memory system
// busy.  A wave alone on its SIMD turns pages over at a rate of its own, set by the load - MFMA -
// softmax - MFMA chain and not by what it has in flight (deep_page_us below: 18.6 GB/s per wave for
// bf16 pages of 8 KiB, 12 GB/s for 4 KiB ones, 7 and 4 GB/s for e4m3 pages of 4 and 2 KiB); past the
// point where the waves together can take about 1.3 times what the memory delivers (6.6 TB/s), every
// further wave only lengthens the queues in front of the memory channels, and the launch gets slower:
// the two-model workload takes 92.6 us with 512 waves, 95-96 with 768, 97.4 with 1024 (and 98.9 with
// 1024 waves that keep 32 KiB in flight each instead of one page pair, 100.9 in the ordinary form).
// Whole CUs' worth of waves only (multiples of 256: with 640 or 896 some CUs hold a wave more than
// others and their waves fall behind: 99.7 / 98.4 us).  Lognormal row lengths, one model, 0.2-2.5 GB
// per launch, ordinary form -> second form: bf16, 128-wide heads 512 waves, 2-17 % faster (more on
// smaller launches); bf16, 64-wide heads 768 waves, 3-13 %; e4m3, 128-wide heads 1024 waves (all the
// form has), 1-12 %; e4m3 with 64-wide heads would need some 2000 such waves and stays with the
// ordinary form (123 against 155 us for 620 MB).  Launches of fewer than 10 240 page units are left to
// the ordinary form as well (within a microsecond either way, mostly in its favour).
constexpr int kDefaultItems = 2048;
constexpr int kDeepMaxItems = 1024, kDeepMinItems = 512, kItemGrain = 256;
constexpr double kDeepMinUnits = 10240.0;
constexpr double kMemBytesPerUs = 6.6e6;       // what the memory system delivers to this kernel at its best
constexpr double kDeepCapacity = 1.3;          // waves' own rate over the memory's, where more waves stop paying
// Smallest share of a wave, in pages.  It only binds in launches too small to give every wave slot a
// share; there the last wave of a (sequence, kv head) merges one partial per piece, one after the
// other, and many small pieces cost more than they gain in parallelism: an eighth of a mean row,
// within 4..16 pages (4 sequences of 2048 tokens: 22.1 us at 4 pages, 16.5-17.3 at 8-16; 8 of 2048:
// 28.2 / 20.4; 16 of 4096 with one kv head: 41.6 / 26.9; rows of 8-16 pages are best left at 4).
constexpr int kDefaultMinShare = 4, kMaxAutoMinShare = 16;
constexpr int kDefaultSegCost = 6;
// Fixed part of a page's cost relative to 0.1 per KiB, in the model that shares the waves of a grouped
// launch out among its models.  Two-model workload (128- and 64-wide heads), second form, 512 waves:
// 95.0 us at 0.8, 92.9 at 1.2, 92.6 at 1.6, 93.4 at 2.0, 94.4 at 2.4, 95.2 at 3.2.
constexpr double kPageCost = 0.8, kDeepPageCost = 1.6;
int g_plan_items = kDefaultItems;     // items of the launch being prepared, all models together
int g_last_items = 0;                 // items of the most recent launch

// Time (us) a wave of the second form, alone on its SIMD, spends on one page.
double deep_page_us(const Model &m) {
    const double page_kib = (double)m.layer_bytes / m.Hkv / 1024.0;
    if (m.dtype == PKV_BF16) return 0.179 * ((g_page_cost >= 0.0 ? g_page_cost : kDeepPageCost) + 0.1 * page_kib);
    return 0.395 + 0.04 * page_kib;
}

// Expected cost of a model's pages, used to share the waves out among the models of a
// grouped launch.  A wave spends a fixed time per page (the load - MFMA - softmax - MFMA
// chain) plus a time per byte, so a model of small pages needs more waves than its bytes
// alone suggest.
double est_bytes(const Model &m, bool own, int batch, int row_stride) {
    const double blocks = own ? (double)m.used_blocks : (double)batch * row_stride;
    if (g_deep_now) return blocks * m.Hkv * deep_page_us(m);
    const double page_kib = (double)m.layer_bytes / m.Hkv / 1024.0;
    return blocks * m.Hkv * ((g_page_cost >= 0.0 ? g_page_cost : kPageCost) + 0.1 * page_kib);
}

// page units (pages plus the allowance per segment) of a model's part of a launch, as far as the host knows
double launch_units(const Model &m, bool own, int batch, int row_stride) {
    const int seg = g_seg_cost >= 0 ? g_seg_cost : kDefaultSegCost;
    return ((own ? (double)m.used_blocks : (double)batch * row_stride) + (double)batch * (seg + 1)) * m.Hkv;
}

// What the host knows of a launch before it is cut: page units, their time in waves of the second form,
// and the bytes they stand for.
struct LaunchLoad {
    double units = 0.0, wave_us = 0.0, bytes = 0.0;
    void add(const Model &m, bool own, int batch, int row_stride) {
        const double u = launch_units(m, own, batch, row_stride);
        units += u;
        wave_us += u * deep_page_us(m);
        bytes += (own ? (double)m.used_blocks : (double)batch * row_stride) * (double)m.layer_bytes;
    }
};

// Chooses the form and the number of items of the launch being prepared.
void plan_launch(const LaunchLoad &l) {
    // waves of the second form that together take kDeepCapacity times what the memory delivers
    const double want = l.bytes > 0.0 ? kDeepCapacity * l.wave_us / (l.bytes / kMemBytesPerUs) : 0.0;
    int n = (int)(want / kItemGrain + 0.5) * kItemGrain;
    const bool fits = n <= kDeepMaxItems + kItemGrain;          // 1280 wanted: 1024 still beat the ordinary form
    n = n < kDeepMinItems ? kDeepMinItems : (n > kDeepMaxItems ? kDeepMaxItems : n);
    if (g_deep_mode >= 0) g_deep_now = g_deep_mode == 1;
    else g_deep_now = g_items == 0 && fits && l.units >= kDeepMinUnits;
    g_plan_items = g_items > 0 ? g_items : (g_deep_now ? n : kDefaultItems);
}

// Everything of a launch descriptor except its split-K workspace.
// cols: MFMA columns per kv head (0 = g: one query token per row); units_hint: upper bound of the
// page units of the launch when the rows are not whole sequences (0 = derive from the blocks in use)
void fill_desc_core(AttnDesc &d, Model &m, int batch, const void *q, const int32_t *table, int row_stride,
                    const int32_t *ctx_lens, float *out, double share_of_launch, int cols = 0, double units_hint = 0.0) {
    Pool &p = g_pools[m.pool];
    const bool own = table == nullptr;
    d.pool_base = p.base + (size_t)m.layer * m.layer_bytes;      // the layer's part of every block
    d.q = (const uint16_t *)q;
    d.table = own ? m.dev.rows : table;
    d.row_stride = own ? m.dev.max_blocks : row_stride;
    d.ctx_lens = ctx_lens;
    d.row_len = own ? m.dev.row_len : nullptr;
    d.out = out;
    d.err = g_err;
    d.safe = g_safe;
    d.frame_bytes = p.frame_bytes;
    d.block_bytes = m.block_bytes;
    d.slots_div = fastdiv_make((uint32_t)m.slots);
    d.max_block_id = (uint32_t)(p.n_frames * m.slots);
    d.batch = batch;
    d.Hq = m.Hq; d.Hkv = m.Hkv; d.g = m.g; d.D = m.D; d.dtype = m.dtype;
    d.vmap = nullptr;
    d.cols = cols > 0 ? cols : m.g;
    d.item_begin = 0;
    d.scale_log2 = (float)(1.4426950408889634 / sqrt((double)m.D));
    if (g_min_share > 0) {
        d.min_share = g_min_share;
    } else {
        const double row_pages = own ? (double)m.used_blocks / batch : (double)row_stride;
        const int eighth = (int)(row_pages / 8.0);
        d.min_share = eighth < kDefaultMinShare ? kDefaultMinShare : (eighth > kMaxAutoMinShare ? kMaxAutoMinShare : eighth);
    }
    d.seg_cost = g_seg_cost >= 0 ? g_seg_cost : kDefaultSegCost;
    // no more items than there can be shares of min_share pages (an empty row counts as one page)
    const double units = units_hint > 0.0 ? units_hint
                                          : ((own ? (double)m.used_blocks : (double)batch * d.row_stride) +
                                             (double)batch * (d.seg_cost + 1)) * m.Hkv;
    double items = g_plan_items * share_of_launch;
    if (items > units / d.min_share) items = units / d.min_share;
    d.n_items = items < 1.0 ? 1 : (int)items;                // never more than the slots in total
    if (d.n_items >= 8) d.n_items &= ~7;                     // whole blocks of eight: one item per XCD
    d.weighted = d.n_items % 8 == 0 ? 1 : 0;
}

// floats of split-K partials a launch of n_items work items needs: two partials per item
size_t ws_floats_for(const Model &m, int n_items, int cols) { return (size_t)2 * n_items * cols * (m.D + 2); }

// The model's own workspace.  It is sized at registration for every launch the default settings can
// produce from the library's table; only a caller's table with more rows than the model has, or a
// work-item count raised through pkv_set_split, makes it grow here (after waiting for the stream).
int ensure_workspace(Model &m, size_t need_floats, size_t n_cnt, size_t slack = 2) {
    if (need_floats > m.ws_floats) {
        HIP_TRY(hipStreamSynchronize(g_stream));
        uc_release(m.ws);
        m.ws_floats = 0;
        m.ws = (float *)uc_alloc(need_floats * sizeof(float) * slack);
        if (!m.ws) return PKV_E_NOMEM;
        m.ws_floats = need_floats * slack;
    }
    if (n_cnt > m.cnt_cap) {
        HIP_TRY(hipStreamSynchronize(g_stream));
        uc_release(m.cnt);
        m.cnt_cap = 0;
        m.cnt = (uint32_t *)uc_alloc(n_cnt * slack * sizeof(uint32_t));
        if (!m.cnt) return PKV_E_NOMEM;
        HIP_TRY(hipMemset(m.cnt, 0, n_cnt * slack * sizeof(uint32_t)));
        m.cnt_cap = n_cnt * slack;
    }
    return PKV_OK;
}

int fill_desc(AttnDesc &d, Model &m, int batch, const void *q, const int32_t *table, int row_stride,
              const int32_t *ctx_lens, float *out, double share_of_launch, int cols = 0, double units_hint = 0.0) {
    fill_desc_core(d, m, batch, q, table, row_stride, ctx_lens, out, share_of_launch, cols, units_hint);
    const int rc = ensure_workspace(m, ws_floats_for(m, d.n_items, d.cols), (size_t)batch * m.Hkv);
    if (rc) return rc;
    d.ws = m.ws;
    d.cnt = m.cnt;
    return PKV_OK;
}

hipEvent_t *next_events() {
    if (!g_timing || (g_launches++ % g_timing) != 0 || g_events_used + 2 > 2 * kMaxTimedLaunches) return nullptr;
    while (g_events.size() < g_events_used + 2) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        g_events.push_back(e);
    }
    hipEvent_t *p = &g_events[g_events_used];
    g_events_used += 2;
    return p;
}

}  // namespace

extern "C" {

int pkv_timing_enable(int every) {
    if (every < 0) return PKV_E_ARG;
    g_timing = every;
    g_launches = 0;
    g_events_used = 0;
    return PKV_OK;
}

long pkv_timing_read(double *attention_ms) {
    HIP_TRY(hipStreamSynchronize(g_stream));
    double a = 0.0;
    for (size_t i = 0; i + 2 <= g_events_used; i += 2) {
        float t = 0.f;
        HIP_TRY(hipEventElapsedTime(&t, g_events[i], g_events[i + 1]));
        a += t;
    }
    if (attention_ms) *attention_ms = a;
    const long n = (long)(g_events_used / 2);
    g_events_used = 0;
    return n;
}

int pkv_set_stream(void *hip_stream) {
    g_stream = (hipStream_t)hip_stream;
    return PKV_OK;
}

const char *pkv_last_error(void) { return g_errbuf; }

static int reconcile_pool(int pool_id);

int pkv_device_errors(void) {
    int rc = lib_init();
    if (rc) return rc;
    uint32_t v = 0;
    HIP_TRY(hipStreamSynchronize(g_stream));
    HIP_TRY(hipMemcpy(&v, g_err, sizeof v, hipMemcpyDeviceToHost));
    if (v) HIP_TRY(hipMemset(g_err, 0, sizeof v));
    v |= g_host_flags;
    g_host_flags = 0;
    if (v & 4u)                     // an enqueued bookkeeping call was refused: the host's estimates are off
        for (int p = 0; p < PKV_MAX_POOLS; ++p)
            if (g_pools[p].live && (rc = reconcile_pool(p)) != PKV_OK) return rc;
    return (int)v;
}

/* ------------------------------------------------------------ XCD weights */

static void normalise_xcd_weights(float *w) {
    for (int pass = 0; pass < 4; ++pass) {          // mean 1 inside the clamp
        double sum = 0.0;
        for (int i = 0; i < 8; ++i) sum += w[i];
        for (int i = 0; i < 8; ++i) {
            w[i] = (float)(w[i] * 8.0 / sum);
            w[i] = w[i] < kXcdWeightMin ? kXcdWeightMin : (w[i] > kXcdWeightMax ? kXcdWeightMax : w[i]);
        }
    }
}

static void fill_tune(AttnTune &t, bool record) {
    double sum = 0.0, acc = 0.0;
    for (int i = 0; i < 8; ++i) sum += g_xcd_w[i];
    t.cum[0] = 0;
    for (int i = 0; i < 8; ++i) {
        acc += g_xcd_w[i];
        t.cum[i + 1] = (uint32_t)(65536.0 * acc / sum + 0.5);
    }
    t.cum[8] = 65536;
    t.stat = record ? g_xcd_stat : nullptr;
}

// one step of the weights from the per-XCD sums of a measured launch (or of several)
static void tune_apply(const uint64_t *tot, bool same_weights) {
    uint64_t d[16];
    for (int i = 0; i < 16; ++i) d[i] = tot[i] - g_tune_last[i];
    for (int i = 0; i < 16; ++i) g_tune_last[i] = tot[i];
    if (!same_weights || (g_tune_left <= 0 && !g_tune_follow)) return;      // measured with weights that have changed since
    double t[8], mean = 0.0;
    for (int i = 0; i < 8; ++i) {
        if (d[2 * i + 1] < 8) return;                    // too few waves on this XCD to judge
        t[i] = (double)d[2 * i] / (double)d[2 * i + 1];
        mean += t[i] / 8.0;
    }
    if (!(mean > 0.0)) return;
    // a wave's time is its share over its XCD's rate: move each weight part of the way to where the
    // times would be equal, and let the next launches correct the rest
    // coarse first, then averaging out the noise, then following slowly
    const double gain = g_tune_left <= 0 ? kSlowTuneGain : (g_tune_done < 8 ? 0.5 : 0.2);
    for (int i = 0; i < 8; ++i) g_xcd_w[i] = (float)(g_xcd_w[i] * pow(mean / t[i], gain));
    normalise_xcd_weights(g_xcd_w);
    if (g_tune_left > 0) {
        ++g_tune_done;
        --g_tune_left;
    }
    ++g_xcd_version;
}

static int tune_setup() {
    if (g_xcd_stat) return PKV_OK;
    HIP_TRY(hipMalloc((void **)&g_xcd_stat, 16 * sizeof(uint64_t)));
    HIP_TRY(hipMemset(g_xcd_stat, 0, 16 * sizeof(uint64_t)));
    HIP_TRY(hipHostMalloc((void **)&g_tune_host, kTuneSlots * 16 * sizeof(uint64_t), hipHostMallocDefault));
    for (int i = 0; i < kTuneSlots; ++i) {
        HIP_TRY(hipEventCreateWithFlags(&g_tune_ev[i], hipEventDisableTiming));
        g_tune_busy[i] = false;
    }
    return PKV_OK;
}

// One attention launch.  While weight updates are owed, a launch that fills the chip is also measured.
static int launch_attention(AttnGroup &grp) {
    // copies of the totals that have arrived meanwhile (never waits)
    for (int i = 0; i < kTuneSlots && g_xcd_stat; ++i)
        if (g_tune_busy[i] && hipEventQuery(g_tune_ev[i]) == hipSuccess) {
            g_tune_busy[i] = false;
            tune_apply(g_tune_host + 16 * i, g_tune_version[i] == g_xcd_version);
        }
    bool measure = g_xcd_stat != nullptr &&
                   ((g_tune_left > 0 && g_tune_measured < kMaxTuneMeasured) || (g_tune_left <= 0 && g_tune_follow));
    int items = 0, slot = -1;
    for (int i = 0; i < grp.n; ++i) {
        items += grp.m[i].n_items;
        measure = measure && grp.m[i].weighted;
    }
    g_last_items = items;
    measure = measure && items >= kMinTuneItems;
    if (measure && g_tune_left <= 0) measure = ++g_tune_tick % kSlowTuneEvery == 0;
    if (measure) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(g_stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) measure = false;
        for (int i = 0; i < kTuneSlots && slot < 0; ++i)
            if (!g_tune_busy[i]) slot = i;
        if (slot < 0) measure = false;                     // all copies still travelling
    }
    fill_tune(grp.tune, measure);
    HIP_TRY(pkv_launch_attention(grp, g_deep_now, g_stream, next_events()));
    if (measure) {
        HIP_TRY(hipMemcpyAsync(g_tune_host + 16 * slot, g_xcd_stat, 16 * sizeof(uint64_t), hipMemcpyDeviceToHost, g_stream));
        HIP_TRY(hipEventRecord(g_tune_ev[slot], g_stream));
        g_tune_busy[slot] = true;
        g_tune_version[slot] = g_xcd_version;
        ++g_tune_measured;
    }
    return PKV_OK;
}

int pkv_set_xcd_weights(const float *w) {
    float v[8];
    for (int i = 0; i < 8; ++i) {
        v[i] = w ? w[i] : 1.f;
        if (!(v[i] > 0.f) || !(v[i] < 1e6f)) return PKV_E_ARG;
    }
    normalise_xcd_weights(v);
    for (int i = 0; i < 8; ++i) g_xcd_w[i] = v[i];
    ++g_xcd_version;
    g_tune_left = 0;              // weights set by hand stay until pkv_tune_xcd asks for tuning again
    g_tune_follow = false;
    return PKV_OK;
}

int pkv_get_xcd_weights(float *w) {
    if (!w) return PKV_E_ARG;
    for (int i = 0; i < 8; ++i) w[i] = g_xcd_w[i];
    return PKV_OK;
}

int pkv_tune_xcd(int updates) {
    if (updates < 0 || updates > 100000) return PKV_E_ARG;
    int rc = lib_init();
    if (rc) return rc;
    g_tune_left = updates;
    g_tune_follow = updates > 0;
    g_tune_done = 0;
    g_tune_measured = 0;
    return PKV_OK;
}

int pkv_set_page_cost(int per_mille) {
    if (per_mille < -1 || per_mille > 100000) return PKV_E_ARG;
    g_page_cost = per_mille < 0 ? -1.0 : per_mille / 1000.0;
    return PKV_OK;
}

int pkv_set_split(int items, int min_share) {
    if (items < 0 || items > (1 << 20) || min_share < 0 || min_share > 4096) return PKV_E_ARG;
    g_items = items;
    g_min_share = min_share;
    return PKV_OK;
}

int pkv_set_kernel_form(int form) {
    if (form < -1 || form > 1) return PKV_E_ARG;
    g_deep_mode = form;
    return PKV_OK;
}

int pkv_last_kernel_form(void) { return g_deep_now ? 1 : 0; }

int pkv_last_launch_items(void) { return g_last_items; }

int pkv_set_segment_cost(int pages) {
    if (pages < -1 || pages > 256) return PKV_E_ARG;
    g_seg_cost = pages;
    return PKV_OK;
}

int pkv_stream_read_probe(size_t bytes, size_t granule_bytes, int iters, double *gbps) {
    if (bytes < (1u << 20) || iters <= 0 || !gbps) return PKV_E_ARG;
    if ((bytes & (bytes - 1)) != 0) return PKV_E_ARG;
    if (granule_bytes != 0 && (granule_bytes < 1024 || (granule_bytes & (granule_bytes - 1)) != 0 || granule_bytes > bytes))
        return PKV_E_ARG;
    int rc = lib_init();
    if (rc) return rc;
    void *buf = nullptr;
    if (hipMalloc(&buf, bytes) != hipSuccess) return PKV_E_NOMEM;
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    HIP_TRY(hipEventCreate(&e1));
    HIP_TRY(hipMemsetAsync(buf, 1, bytes, g_stream));
    HIP_TRY(pkv_launch_stream_read(buf, bytes, granule_bytes, g_err, g_stream));       // warm-up
    HIP_TRY(hipEventRecord(e0, g_stream));
    for (int i = 0; i < iters; ++i) HIP_TRY(pkv_launch_stream_read(buf, bytes, granule_bytes, g_err, g_stream));
    HIP_TRY(hipEventRecord(e1, g_stream));
    HIP_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
    *gbps = (double)bytes * iters / (ms * 1e-3) / 1e9;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(buf);
    return PKV_OK;
}


int pkv_debug_fail_frame_map(int after) {
    if (after < -1) return PKV_E_ARG;
    g_fail_map_after = after;
    return PKV_OK;
}

uint32_t pkv_debug_fastdiv(uint32_t n, uint32_t d) {
    if (d == 0) return 0;
    return fastdiv_div(n, fastdiv_make(d));
}

/* ------------------------------------------------------------------ pool */

int pool_create_ex(size_t bytes, int page_tokens, size_t frame_bytes, void *device_base) {
    if (page_tokens <= 0 || frame_bytes == 0 || bytes < frame_bytes) return PKV_E_ARG;
    if (frame_bytes % 256 != 0 || ((uintptr_t)device_base & 255) != 0) return PKV_E_ARG;
    const int64_t n_frames = (int64_t)(bytes / frame_bytes);
    if (n_frames > 0x7fffffffLL / 4) return PKV_E_ARG;
    int rc = lib_init();
    if (rc) return rc;
    int id = -1;
    for (int i = 0; i < PKV_MAX_POOLS; ++i)
        if (!g_pools[i].live) { id = i; break; }
    if (id < 0) return PKV_E_NOMEM;
    Pool p;
    p.bytes = bytes; p.frame_bytes = frame_bytes; p.T = page_tokens; p.n_frames = n_frames;
    if (device_base) {
        p.base = (uint8_t *)device_base;
    } else {
        hipError_t e = hipMalloc((void **)&p.base, (size_t)n_frames * frame_bytes);
        if (e != hipSuccess) { fail_hip(e, "hipMalloc(pool)"); return PKV_E_NOMEM; }
        p.own_base = true;
    }
    p.dev.n_frames = n_frames;
    hipError_t e = hipMalloc((void **)&p.dev.owner, sizeof(int32_t) * n_frames);
    if (e == hipSuccess) e = hipMalloc((void **)&p.dev.free_stack, sizeof(uint32_t) * n_frames);
    if (e == hipSuccess) e = hipMalloc((void **)&p.dev.pos, sizeof(int32_t) * n_frames);
    if (e == hipSuccess) e = hipMalloc((void **)&p.dev.n_free, sizeof(int64_t));
    if (e == hipSuccess) e = pkv_launch_pool_init(p.dev, nullptr, g_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(g_stream);
    if (e != hipSuccess) {
        (void)hipFree(p.dev.owner); (void)hipFree(p.dev.free_stack); (void)hipFree(p.dev.pos); (void)hipFree(p.dev.n_free);
        if (p.own_base) (void)hipFree(p.base);
        return fail_hip(e, "pool_create");
    }
    p.live = true;
    p.n_free = n_frames;
    g_pools[id] = p;
    g_last_pool = id;
    return id;
}

/* ------------------------------------------------------------ elastic pools */

static hipMemAllocationProp device_memory_prop() {
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    int dev = 0;
    (void)hipGetDevice(&dev);
    prop.location.id = dev;
    return prop;
}

static hipError_t frame_map(Elastic &el, uint32_t f, hipMemGenericAllocationHandle_t h) {
    void *at = el.base + (size_t)f * el.frame_bytes;
    hipError_t e = hipMemMap(at, el.frame_bytes, 0, h, 0);
    if (e != hipSuccess) return e;
    hipMemAccessDesc acc = {};
    acc.location.type = hipMemLocationTypeDevice;
    acc.location.id = el.device;
    acc.flags = hipMemAccessFlagsProtReadWrite;
    e = hipMemSetAccess(at, el.frame_bytes, &acc, 1);
    if (e != hipSuccess) (void)hipMemUnmap(at, el.frame_bytes);
    return e;
}

static hipError_t frame_create(Elastic &el, hipMemGenericAllocationHandle_t *h) {
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = el.device;
    return hipMemCreate(h, el.frame_bytes, &prop, 0);
}

// The pre-allocation thread.  It holds the lock only to choose its next task and to publish the outcome;
// the driver calls (a mapping costs tens of microseconds, an unmapping a quarter of a millisecond) run
// with the lock released, the frame marked F_MAPPING / F_UNMAPPING meanwhile.
static void elastic_worker(Elastic *el) {
    (void)hipSetDevice(el->device);
    std::unique_lock<std::mutex> lk(el->mu);
    while (!el->stop) {
        const uint64_t gen = el->changes;
        const size_t n = el->stack.size();
        const size_t top_from = n > el->target ? n - el->target : 0;      // positions >= top_from form the buffer
        if (el->low_water > n) el->low_water = n;
        // 1. a frame of the buffer that has no memory yet (nearest to the top first: it is taken first)
        long map_at = -1;
        for (size_t i = n; i-- > top_from;)
            if (el->state[el->stack[i]] == F_UNMAPPED) { map_at = (long)i; break; }
        if (map_at >= 0) {
            const uint32_t f = el->stack[(size_t)map_at];
            hipMemGenericAllocationHandle_t h{};
            el->state[f] = F_MAPPING;
            el->idle = false;
            lk.unlock();
            hipError_t e = frame_create(*el, &h);
            if (e == hipSuccess && (e = frame_map(*el, f, h)) != hipSuccess) (void)hipMemRelease(h);
            lk.lock();
            if (e == hipSuccess) {
                el->handle[f] = h;
                el->state[f] = F_MAPPED;
                el->mapped_frames++;
                el->mapped_free++;          // (a model that took the frame meanwhile waits for this state and corrects the count)
                if ((size_t)map_at < el->low_water) el->low_water = (size_t)map_at;
                el->done.notify_all();
                continue;
            }
            // no memory for the buffer right now: leave the frame as it was and rest until something changes
            el->state[f] = F_UNMAPPED;
        } else {
            // 2. a free frame below the buffer that still has memory
            long unmap_at = -1;
            while (el->low_water < top_from) {
                if (el->state[el->stack[el->low_water]] == F_MAPPED) { unmap_at = (long)el->low_water; break; }
                el->low_water++;
            }
            if (unmap_at >= 0) {
                const uint32_t f = el->stack[(size_t)unmap_at];
                const hipMemGenericAllocationHandle_t h = el->handle[f];
                el->state[f] = F_UNMAPPING;
                el->idle = false;
                lk.unlock();
                (void)hipMemUnmap(el->base + (size_t)f * el->frame_bytes, el->frame_bytes);
                (void)hipMemRelease(h);
                lk.lock();
                el->state[f] = F_UNMAPPED;
                el->mapped_frames--;
                el->mapped_free--;
                el->done.notify_all();
                continue;
            }
        }
        el->seen = gen;
        el->idle = true;
        el->done.notify_all();
        el->work.wait(lk, [&] { return el->stop || el->changes != el->seen; });
    }
}

// A model has acquired frame f (already popped from the copy of the stack): make sure memory backs it
// before the call returns.  Called with the lock held.
static int elastic_acquire(Elastic &el, uint32_t f, std::unique_lock<std::mutex> &lk) {
    while (el.state[f] == F_MAPPING || el.state[f] == F_UNMAPPING) el.done.wait(lk);
    if (el.state[f] == F_MAPPED) {
        el.mapped_free--;
        return PKV_OK;
    }
    if (g_fail_map_after >= 0 && g_fail_map_after-- == 0) {
        snprintf(g_errbuf, sizeof g_errbuf, "frame %u: mapping refused (pkv_debug_fail_frame_map)", f);
        return PKV_E_NOMEM;
    }
    hipMemGenericAllocationHandle_t h{};
    el.state[f] = F_MAPPING;
    lk.unlock();
    hipError_t e = frame_create(el, &h);
    int rc = PKV_OK;
    if (e != hipSuccess) {
        fail_hip(e, "hipMemCreate(frame)");
        rc = PKV_E_NOMEM;
    } else if ((e = frame_map(el, f, h)) != hipSuccess) {
        (void)hipMemRelease(h);
        fail_hip(e, "hipMemMap(frame)");
        rc = PKV_E_DEVICE;
    }
    lk.lock();
    if (rc == PKV_OK) {
        el.handle[f] = h;
        el.state[f] = F_MAPPED;
        el.mapped_frames++;
    } else {
        el.state[f] = F_UNMAPPED;
    }
    el.done.notify_all();
    return rc;
}

// wait until the pre-allocation thread has dealt with every change made so far (it rests early only if
// the driver has no memory for the buffer)
static void elastic_settle(Elastic &el) {
    std::unique_lock<std::mutex> lk(el.mu);
    el.work.notify_all();
    el.done.wait(lk, [&] { return el.idle && el.seen == el.changes; });
}

// callers, with the lock held, after any change of the stack copy or of the target
static void elastic_changed(Elastic &el) {
    ++el.changes;
    el.work.notify_one();
}

static void elastic_shutdown(Pool &p) {
    Elastic *el = p.el;
    if (!el) return;
    {
        std::lock_guard<std::mutex> g(el->mu);
        el->stop = true;
    }
    el->work.notify_all();
    if (el->worker.joinable()) el->worker.join();
    for (size_t f = 0; f < el->state.size(); ++f)
        if (el->state[f] == F_MAPPED) {
            (void)hipMemUnmap(el->base + f * el->frame_bytes, el->frame_bytes);
            (void)hipMemRelease(el->handle[f]);
        }
    delete el;
    p.el = nullptr;
}

int pool_create_elastic(size_t bytes, int page_tokens, size_t frame_bytes) {
    if (page_tokens <= 0 || frame_bytes == 0 || bytes < frame_bytes) return PKV_E_ARG;
    int rc = lib_init();
    if (rc) return rc;
    const hipMemAllocationProp prop = device_memory_prop();
    size_t gran = 0;
    hipError_t e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum);
    if (e != hipSuccess) { fail_hip(e, "hipMemGetAllocationGranularity"); return PKV_E_UNSUPPORTED; }
    if (gran == 0 || frame_bytes % gran != 0 || frame_bytes % 256 != 0) return PKV_E_SHAPE;
    const int64_t n_frames = (int64_t)(bytes / frame_bytes);
    void *va = nullptr;
    e = hipMemAddressReserve(&va, (size_t)n_frames * frame_bytes, 0, nullptr, 0);
    if (e != hipSuccess) { fail_hip(e, "hipMemAddressReserve"); return PKV_E_NOMEM; }
    const int id = pool_create_ex((size_t)n_frames * frame_bytes, page_tokens, frame_bytes, va);
    if (id < 0) {
        (void)hipMemAddressFree(va, (size_t)n_frames * frame_bytes);
        return id;
    }
    Pool &p = g_pools[id];
    p.elastic = true;
    Elastic *el = new Elastic;
    (void)hipGetDevice(&el->device);
    el->base = p.base;
    el->frame_bytes = frame_bytes;
    el->state.assign((size_t)n_frames, F_UNMAPPED);
    el->handle.assign((size_t)n_frames, hipMemGenericAllocationHandle_t{});
    el->stack.resize((size_t)n_frames);
    for (int64_t i = 0; i < n_frames; ++i) el->stack[(size_t)i] = (uint32_t)(n_frames - 1 - i);   // frame 0 on top
    p.el = el;
    el->worker = std::thread(elastic_worker, el);
    static bool at_exit = false;
    if (!at_exit) {                      // a process that ends with elastic pools alive: stop their threads before the runtime goes
        at_exit = true;
        atexit([] {
            for (int i = 0; i < PKV_MAX_POOLS; ++i) {
                Elastic *e = g_pools[i].live ? g_pools[i].el : nullptr;
                if (!e) continue;
                {
                    std::lock_guard<std::mutex> g(e->mu);
                    e->stop = true;
                }
                e->work.notify_all();
                if (e->worker.joinable()) e->worker.join();
            }
        });
    }
    return id;
}

int pool_set_prealloc(int pool, long frames) {
    Pool *p = get_pool(pool);
    if (!p) return PKV_E_HANDLE;
    if (!p->elastic || frames < 0 || frames > p->n_frames) return PKV_E_ARG;
    Elastic &el = *p->el;
    {
        std::lock_guard<std::mutex> g(el.mu);
        el.target = (size_t)frames;
        el.low_water = 0;
        elastic_changed(el);
    }
    elastic_settle(el);
    std::lock_guard<std::mutex> g(el.mu);
    return (int)el.mapped_free;
}

int pool_prealloc_wait(int pool) {
    Pool *p = get_pool(pool);
    if (!p) return PKV_E_HANDLE;
    if (!p->elastic) return 0;
    elastic_settle(*p->el);
    std::lock_guard<std::mutex> g(p->el->mu);
    return (int)p->el->mapped_free;
}

int pool_create(size_t bytes, int page_tokens) {
    return pool_create_ex(bytes, page_tokens, (size_t)2 << 20, nullptr);
}

int pool_destroy(int pool) {
    Pool *p = get_pool(pool);
    if (!p) return PKV_E_HANDLE;
    for (int m = 0; m < PKV_MAX_MODELS; ++m)
        if (g_models[m].live && g_models[m].pool == pool) return PKV_E_BUSY;
    HIP_TRY(hipStreamSynchronize(g_stream));
    (void)hipFree(p->dev.owner); (void)hipFree(p->dev.free_stack); (void)hipFree(p->dev.pos); (void)hipFree(p->dev.n_free);
    if (p->own_base) (void)hipFree(p->base);
    if (p->elastic) {
        const size_t range = (size_t)p->n_frames * p->frame_bytes;
        uint8_t *base = p->base;
        elastic_shutdown(*p);
        (void)hipMemAddressFree(base, range);
    }
    *p = Pool{};
    if (g_last_pool == pool) g_last_pool = -1;
    return PKV_OK;
}

int pool_seed_free_order(int pool, const uint32_t *perm, size_t n) {
    Pool *p = get_pool(pool);
    if (!p) return PKV_E_HANDLE;
    if (!perm || (int64_t)n != p->n_frames) return PKV_E_ARG;
    int rcs = reconcile_pool(pool);
    if (rcs) return rcs;
    for (int m = 0; m < PKV_MAX_MODELS; ++m)      // only while every frame is still free
        if (g_models[m].live && g_models[m].pool == pool && g_models[m].owned != 0) return PKV_E_ARG;
    std::vector<uint8_t> seen(n, 0);
    for (size_t i = 0; i < n; ++i) {
        if (perm[i] >= n || seen[perm[i]]) return PKV_E_ARG;
        seen[perm[i]] = 1;
    }
    uint32_t *dperm = nullptr;
    HIP_TRY(hipMalloc((void **)&dperm, sizeof(uint32_t) * n));
    hipError_t e = hipMemcpyAsync(dperm, perm, sizeof(uint32_t) * n, hipMemcpyHostToDevice, g_stream);
    if (e == hipSuccess) e = pkv_launch_pool_init(p->dev, dperm, g_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(g_stream);
    (void)hipFree(dperm);
    if (e != hipSuccess) return fail_hip(e, "pool_seed_free_order");
    if (p->elastic) {                   // the host's copy of the free stack follows: perm[0] on top
        std::lock_guard<std::mutex> g(p->el->mu);
        for (size_t i = 0; i < n; ++i) p->el->stack[n - 1 - i] = perm[i];
        p->el->low_water = 0;
        elastic_changed(*p->el);
    }
    return PKV_OK;
}

/* ----------------------------------------------------------------- model */

int model_register_ex(int pool, int q_heads, int kv_heads, int head_dim, int dtype, int max_seqs,
                      int max_blocks_per_seq) {
    return model_register_layers(pool, q_heads, kv_heads, head_dim, dtype, max_seqs, max_blocks_per_seq, 1);
}

int pkv_set_layer(int model, int layer) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (layer < 0 || layer >= m->L) return PKV_E_ARG;
    m->layer = layer;
    return PKV_OK;
}

int model_register_layers(int pool, int q_heads, int kv_heads, int head_dim, int dtype, int max_seqs,
                          int max_blocks_per_seq, int n_layers) {
    Pool *p = get_pool(pool);
    if (!p) return PKV_E_HANDLE;
    if (q_heads <= 0 || kv_heads <= 0 || head_dim <= 0 || max_seqs <= 0 || max_blocks_per_seq <= 0 ||
        n_layers <= 0)
        return PKV_E_ARG;
    if (dtype != PKV_BF16 && dtype != PKV_E4M3) return PKV_E_ARG;
    if (max_seqs > PKV_MAX_SEQS || max_blocks_per_seq > PKV_MAX_ROW_BLOCKS) return PKV_E_ARG;
    if (q_heads % kv_heads != 0) return PKV_E_SHAPE;
    const size_t e = dtype == PKV_BF16 ? 2 : 1;
    size_t block_bytes = (size_t)2 * p->T * kv_heads * head_dim * e;
    if (dtype == PKV_E4M3) {
        if ((size_t)kv_heads * 2 * sizeof(float) > PKV_FP8_HEADER) return PKV_E_SHAPE;
        block_bytes += PKV_FP8_HEADER;
    }
    const size_t layer_bytes = block_bytes;
    block_bytes *= (size_t)n_layers;
    const size_t slots = p->frame_bytes / block_bytes;
    if (slots == 0) return PKV_E_SHAPE;
    // what the gfx950 kernels are built for
    if (p->T != 16 || (head_dim != 64 && head_dim != 128) || q_heads / kv_heads > 16) return PKV_E_UNSUPPORTED;
    int id = -1;
    for (int i = 0; i < PKV_MAX_MODELS; ++i)
        if (!g_models[i].live) { id = i; break; }
    if (id < 0) return PKV_E_NOMEM;
    Model m;
    m.pool = pool;
    m.Hq = q_heads; m.Hkv = kv_heads; m.D = head_dim; m.dtype = dtype; m.g = q_heads / kv_heads;
    m.L = n_layers;
    m.layer_bytes = layer_bytes;
    m.block_bytes = block_bytes;
    m.slots = (int)slots;
    m.row_len.assign(max_seqs, 0);
    ModelDev &d = m.dev;
    d.model_id = id;
    d.slots = (int)slots;
    d.wpf = (int)((slots + 31) / 32);
    d.max_seqs = max_seqs;
    d.max_blocks = max_blocks_per_seq;
    d.page_tokens = p->T;
    const int64_t nf = p->n_frames;
    hipError_t err = hipMalloc((void **)&d.frames, sizeof(uint32_t) * nf);
    if (err == hipSuccess) err = hipMalloc((void **)&d.bits, sizeof(uint32_t) * nf * d.wpf);
    if (err == hipSuccess) err = hipMalloc((void **)&d.mark, (size_t)nf);
    if (err == hipSuccess) err = hipMalloc((void **)&d.rows, sizeof(int32_t) * (size_t)max_seqs * max_blocks_per_seq);
    if (err == hipSuccess) err = hipMalloc((void **)&d.row_len, sizeof(int32_t) * max_seqs);
    if (err == hipSuccess) err = hipMalloc((void **)&d.counters, sizeof(int64_t) * 2);
    if (err == hipSuccess) err = hipMemsetAsync(d.rows, 0, sizeof(int32_t) * (size_t)max_seqs * max_blocks_per_seq, g_stream);
    if (err == hipSuccess) err = hipMemsetAsync(d.row_len, 0, sizeof(int32_t) * max_seqs, g_stream);
    if (err == hipSuccess) err = hipMemsetAsync(d.counters, 0, sizeof(int64_t) * 2, g_stream);
    if (err == hipSuccess) err = hipStreamSynchronize(g_stream);
    if (err != hipSuccess) {
        free_model_dev(m);
        fail_hip(err, "model_register");
        return PKV_E_NOMEM;
    }
    // the split-K workspace of decode attention, for the largest launch the default settings give
    // this model, so that decode_attention* neither waits nor allocates (graph capture needs no
    // priming launch)
    {
        const int rc = ensure_workspace(m, ws_floats_for(m, kDefaultItems, m.g), (size_t)max_seqs * kv_heads, 1);
        if (rc) {
            free_model_dev(m);
            return rc;
        }
    }
    m.live = true;
    g_models[id] = m;
    return id;
}

int model_register(int q_heads, int kv_heads, int head_dim, int dtype) {
    if (g_last_pool < 0) return PKV_E_HANDLE;
    return model_register_ex(g_last_pool, q_heads, kv_heads, head_dim, dtype, 256, 2048);
}

int model_unregister(int model) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    int rcs = reconcile_pool(m->pool);
    if (rcs) return rcs;
    if (m->owned != 0) return PKV_E_BUSY;
    HIP_TRY(hipStreamSynchronize(g_stream));
    free_model_dev(*m);
    *m = Model{};
    return PKV_OK;
}

/* --------------------------------------------------------------- balloon */

// Bring the host's shadows of a pool and its models back in line with the device: waits for every
// bookkeeping call still in flight, then reads the counts the kernels keep.
static int reconcile_pool(int pool_id) {
    Pool &p = g_pools[pool_id];
    bool any = false;
    for (int id = 0; id < PKV_MAX_MODELS; ++id) any |= g_models[id].live && g_models[id].pool == pool_id && g_models[id].stale;
    if (!any) return PKV_OK;
    for (int i = 0; i < kTickets; ++i)
        if (g_tickets[i].id >= 0 && g_res[i].value == kPending) HIP_TRY(hipStreamSynchronize(g_tickets[i].stream));
    HIP_TRY(hipMemcpy(&p.n_free, p.dev.n_free, sizeof(int64_t), hipMemcpyDeviceToHost));
    for (int id = 0; id < PKV_MAX_MODELS; ++id) {
        Model &m = g_models[id];
        if (!m.live || m.pool != pool_id || !m.stale) continue;
        int64_t cnt[2];
        HIP_TRY(hipMemcpy(cnt, m.dev.counters, sizeof cnt, hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(m.row_len.data(), m.dev.row_len, sizeof(int32_t) * m.row_len.size(), hipMemcpyDeviceToHost));
        m.owned = cnt[0];
        m.used_blocks = cnt[0] * m.slots - cnt[1];
        m.stale = false;
    }
    return PKV_OK;
}

// balloon_resize on an ordinary pool: one kernel that decides the direction itself.
// sticky: a refusal also raises bit 2 of the device flags (the enqueue-only forms; the caller of a
// synchronous form gets the code itself)
static int enqueue_resize(Model &m, long pages, bool sticky = false) {
    Pool &p = g_pools[m.pool];
    const int slot = take_ticket();
    hipError_t e = pkv_launch_resize(p.dev, m.dev, pages, &g_res[slot], sticky ? g_err : nullptr, g_stream);
    if (e != hipSuccess) {
        g_res[slot].value = fail_hip(e, "balloon_resize launch");
        return slot;
    }
    return slot;
}

long balloon_resize(int model, long pages) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (pages < 0) return PKV_E_ARG;
    Pool &p = g_pools[m->pool];
    if (pages > p.n_frames) return PKV_E_NOMEM;
    if (!p.elastic) {
        const int64_t r = wait_ticket(enqueue_resize(*m, pages));
        if (r >= 0) {
            p.n_free -= r - m->owned;
            m->owned = r;
        }
        return (long)r;
    }
    // elastic pool: the frames that change hands are mapped / given back by the host, which therefore
    // needs to know exactly what the model owned before
    int rc = reconcile_pool(m->pool);
    if (rc) return rc;
    const int64_t before = m->owned;
    if (pages == before) return (long)before;
    const int64_t r = wait_ticket(enqueue_resize(*m, pages));
    if (r < 0) return (long)r;
    // the bookkeeping has changed: bring the shadows along before any mapping work, so that a failure
    // below cannot leave them behind the device's state
    const int64_t n_free_before = p.n_free;
    p.n_free -= r - before;
    m->owned = r;
    Elastic &el = *p.el;
    if (r > before) {
        // the kernel chose the frames (the top of the free stack, topmost first: they are the new tail of the
        // model's frame list); memory must back them before anyone can place a block there.  Those that
        // waited in the buffer have it already.
        const size_t k = (size_t)(r - before);
        std::vector<uint32_t> got(k);
        hipError_t e = hipMemcpy(got.data(), m->dev.frames + before, k * sizeof(uint32_t), hipMemcpyDeviceToHost);
        int fail = e == hipSuccess ? PKV_OK : fail_hip(e, "balloon_resize: reading the acquired frames");
        std::unique_lock<std::mutex> lk(el.mu);
        size_t backed = 0;
        if (fail == PKV_OK) {
            for (size_t i = 0; i < k; ++i) {
                if (el.stack.empty() || el.stack.back() != got[i]) return PKV_E_INTERNAL;     // the copy of the stack is off
                el.stack.pop_back();
            }
            for (; backed < k; ++backed)
                if ((fail = elastic_acquire(el, got[backed], lk)) != PKV_OK) break;
            if (fail == PKV_OK) {
                elastic_changed(el);
                return (long)r;
            }
        }
        // No memory for a frame (or the list could not be read): undo the whole inflate, or kernels could
        // be pointed at an address nothing backs.  The frames just taken are the model's newest and hold
        // no block, so a deflate to the old size hands back exactly them, in the order that restores the
        // free stack (the newest first, so the one taken first ends on top again).
        lk.unlock();
        const int64_t back = wait_ticket(enqueue_resize(*m, before));
        if (back >= 0) {
            p.n_free -= back - m->owned;
            m->owned = back;
        }
        lk.lock();
        if (e == hipSuccess && back == before) {
            if (el.stack.size() < el.low_water) el.low_water = el.stack.size();      // mapped frames arrive from here up
            for (size_t i = k; i-- > 0;) el.stack.push_back(got[i]);
            el.mapped_free += (int64_t)backed;         // those that got their memory keep it, as free frames of the buffer
            elastic_changed(el);
        }
        return back == before ? fail : PKV_E_INTERNAL;
    }
    // a deflate: the frames given back are the new top of the free stack, in the order the kernel pushed them.
    // They keep their memory for now (nothing is unmapped inside this call): the top ones are the buffer, the
    // pre-allocation thread takes the memory of those that lie deeper.  Nothing refers to them any more: they
    // held no block, and the work enqueued before the deflate has ended (the call above waited for its kernel).
    const size_t k = (size_t)(before - r);
    std::vector<uint32_t> gone(k);
    HIP_TRY(hipMemcpy(gone.data(), p.dev.free_stack + n_free_before, k * sizeof(uint32_t), hipMemcpyDeviceToHost));
    std::lock_guard<std::mutex> g(el.mu);
    if (el.stack.size() < el.low_water) el.low_water = el.stack.size();              // mapped frames arrive from here up
    for (size_t j = 0; j < k; ++j) el.stack.push_back(gone[j]);
    el.mapped_free += (int64_t)k;
    elastic_changed(el);
    return (long)r;
}

int balloon_resize_enqueue(int model, long pages) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (pages < 0) return PKV_E_ARG;
    Pool &p = g_pools[m->pool];
    if (p.elastic) {
        // mapping and unmapping frames is host work that needs the kernel's choice: done at once
        return ticket_handle(finished_ticket(balloon_resize(model, pages)));
    }
    if (pages > p.n_frames) {
        g_host_flags |= 4u;
        return ticket_handle(finished_ticket(PKV_E_NOMEM));
    }
    const int slot = enqueue_resize(*m, pages, true);
    // estimate: the call succeeds in full
    p.n_free -= pages - m->owned;
    m->owned = pages;
    m->stale = true;
    return ticket_handle(slot);
}

// checks of a reserve list that need no device state, in the order of the sequential definition
static int check_reserve_list(const Model &m, int T, int n, const int32_t *seqs, const int32_t *ctx_lens) {
    for (int i = 0; i < n; ++i) {
        if (seqs[i] < 0 || seqs[i] >= m.dev.max_seqs || ctx_lens[i] < 0) return PKV_E_ARG;
        if (((int64_t)ctx_lens[i] + T - 1) / T > m.dev.max_blocks) return PKV_E_RANGE;
    }
    return PKV_OK;
}

static int enqueue_reserve(Model &m, int n, const int32_t *seqs, const int32_t *ctx_lens, bool sticky = false) {
    Pool &p = g_pools[m.pool];
    const int slot = take_ticket();
    int32_t *ops = ticket_ops(slot);
    memcpy(ops, seqs, sizeof(int32_t) * n);
    memcpy(ops + n, ctx_lens, sizeof(int32_t) * n);
    // What an entry's row holds before it, as far as the list alone decides: the largest want among the
    // earlier entries of the same sequence (the list has passed check_reserve_list).  The kernel takes the
    // larger of this and the row's length on the device, which leaves it nothing to order among entries.
    int32_t *earlier = ops + 2 * n;
    if (m.list_max.size() < (size_t)m.dev.max_seqs) m.list_max.assign((size_t)m.dev.max_seqs, 0);
    for (int i = 0; i < n; ++i) {
        const int want = (int)(((int64_t)ctx_lens[i] + p.T - 1) / p.T);
        int32_t &seen = m.list_max[(size_t)seqs[i]];
        earlier[i] = seen;
        if (want > seen) seen = want;
    }
    for (int i = 0; i < n; ++i) m.list_max[(size_t)seqs[i]] = 0;
    hipError_t e = pkv_launch_reserve(p.dev, m.dev, n, ops, &g_res[slot], sticky ? g_err : nullptr, g_stream);
    if (e != hipSuccess) g_res[slot].value = fail_hip(e, "seq_reserve_batch launch");
    return slot;
}

// the effect of a reserve list that succeeds as a whole on the shadows; returns the blocks added
static int64_t shadow_reserve(Model &m, int T, int n, const int32_t *seqs, const int32_t *ctx_lens) {
    int64_t added = 0;
    for (int i = 0; i < n; ++i) {
        const int want = (int)(((int64_t)ctx_lens[i] + T - 1) / T);
        if (want > m.row_len[seqs[i]]) {
            added += want - m.row_len[seqs[i]];
            m.row_len[seqs[i]] = want;
        }
    }
    m.used_blocks += added;
    return added;
}

int seq_reserve_batch(int model, int n, const int32_t *seqs, const int32_t *ctx_lens) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (n < 0 || n > PKV_MAX_BATCH_OPS || (n > 0 && (!seqs || !ctx_lens))) return PKV_E_ARG;
    if (n == 0) return 0;
    Pool &p = g_pools[m->pool];
    int rc = check_reserve_list(*m, p.T, n, seqs, ctx_lens);
    if (rc) return rc;
    const int64_t r = wait_ticket(enqueue_reserve(*m, n, seqs, ctx_lens));
    if (r >= 0) shadow_reserve(*m, p.T, n, seqs, ctx_lens);   // the call succeeded as a whole: replay its effect
    return (int)r;
}

int seq_reserve_batch_enqueue(int model, int n, const int32_t *seqs, const int32_t *ctx_lens) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (n < 0 || n > PKV_MAX_BATCH_OPS || (n > 0 && (!seqs || !ctx_lens))) return PKV_E_ARG;
    if (n == 0) return ticket_handle(finished_ticket(0));
    Pool &p = g_pools[m->pool];
    int rc = check_reserve_list(*m, p.T, n, seqs, ctx_lens);
    if (rc) {                                                 // refused before anything was enqueued
        g_host_flags |= 4u;
        return ticket_handle(finished_ticket(rc));
    }
    const int slot = enqueue_reserve(*m, n, seqs, ctx_lens, true);
    shadow_reserve(*m, p.T, n, seqs, ctx_lens);               // estimate: the call succeeds
    m->stale = true;
    return ticket_handle(slot);
}

int seq_reserve(int model, int seq, int ctx_len) {
    const int32_t s = seq, c = ctx_len;
    return seq_reserve_batch(model, 1, &s, &c);
}

static int enqueue_release(Model &m, int n, const int32_t *seqs, bool sticky = false) {
    Pool &p = g_pools[m.pool];
    const int slot = take_ticket();
    int32_t *ops = ticket_ops(slot);
    memcpy(ops, seqs, sizeof(int32_t) * n);
    hipError_t e = pkv_launch_release(p.dev, m.dev, n, ops, &g_res[slot], sticky ? g_err : nullptr, g_stream);
    if (e != hipSuccess) g_res[slot].value = fail_hip(e, "seq_release launch");
    return slot;
}

static void shadow_release(Model &m, int n, const int32_t *seqs) {
    for (int i = 0; i < n; ++i) {
        m.used_blocks -= m.row_len[seqs[i]];
        m.row_len[seqs[i]] = 0;
    }
}

int seq_release_batch(int model, int n, const int32_t *seqs) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (n < 0 || n > PKV_MAX_SEQS || (n > 0 && !seqs)) return PKV_E_ARG;
    for (int i = 0; i < n; ++i)
        if (seqs[i] < 0 || seqs[i] >= m->dev.max_seqs) return PKV_E_ARG;
    if (n == 0) return 0;
    const int64_t r = wait_ticket(enqueue_release(*m, n, seqs));
    if (r >= 0) shadow_release(*m, n, seqs);
    return (int)r;
}

int seq_release_batch_enqueue(int model, int n, const int32_t *seqs) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (n < 0 || n > PKV_MAX_SEQS || (n > 0 && !seqs)) return PKV_E_ARG;
    for (int i = 0; i < n; ++i)
        if (seqs[i] < 0 || seqs[i] >= m->dev.max_seqs) return PKV_E_ARG;
    if (n == 0) return ticket_handle(finished_ticket(0));
    const int slot = enqueue_release(*m, n, seqs, true);
    shadow_release(*m, n, seqs);
    m->stale = true;
    return ticket_handle(slot);
}

int seq_release(int model, int seq) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (seq < 0 || seq >= m->dev.max_seqs) return PKV_E_ARG;
    if (!m->stale && m->row_len[seq] == 0) return 0;
    const int32_t s = seq;
    return seq_release_batch(model, 1, &s);
}

long pkv_ticket_result(int ticket) {
    if (ticket < 0) return PKV_E_ARG;
    for (int slot = 0; slot < kTickets; ++slot)
        if (g_tickets[slot].id >= 0 && (int)(g_tickets[slot].id & 0x7fffffff) == ticket) return (long)wait_ticket(slot);
    return PKV_E_RANGE;        // older than the ring remembers
}

const int32_t *model_block_table(int model, int *row_stride) {
    Model *m = get_model(model);
    if (!m) return nullptr;
    if (row_stride) *row_stride = m->dev.max_blocks;
    return m->dev.rows;
}

/* ---------------------------------------------------------------- KV data */

int kv_write(int model, int seq, int tok_begin, int n_tok, const void *k, const void *v, const float *k_scale,
             const float *v_scale) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (seq < 0 || seq >= m->dev.max_seqs || tok_begin < 0 || n_tok < 0) return PKV_E_ARG;
    if (n_tok == 0) return 0;
    if (!k || !v) return PKV_E_ARG;
    if (m->dtype == PKV_E4M3 && (!k_scale || !v_scale)) return PKV_E_ARG;
    Pool &p = g_pools[m->pool];
    if (m->stale) {                 // the range check below needs the row's true length
        int rcs = reconcile_pool(m->pool);
        if (rcs) return rcs;
    }
    if (((int64_t)tok_begin + n_tok + p.T - 1) / p.T > m->row_len[seq]) return PKV_E_RANGE;
    AttnDesc d{};
    d.pool_base = p.base + (size_t)m->layer * m->layer_bytes;
    d.table = m->dev.rows;
    d.row_stride = m->dev.max_blocks;
    d.frame_bytes = p.frame_bytes;
    d.block_bytes = m->block_bytes;
    d.slots_div = fastdiv_make((uint32_t)m->slots);
    d.Hq = m->Hq; d.Hkv = m->Hkv; d.g = m->g; d.D = m->D; d.dtype = m->dtype;
    HIP_TRY(pkv_launch_kv_write(d, seq, tok_begin, n_tok, k, v, k_scale, v_scale, p.T, g_stream));
    return n_tok;
}

// the part of a descriptor that addressing a model's own blocks needs
static void fill_addressing(AttnDesc &d, const Model &m) {
    const Pool &p = g_pools[m.pool];
    d.pool_base = p.base + (size_t)m.layer * m.layer_bytes;
    d.table = m.dev.rows;
    d.row_stride = m.dev.max_blocks;
    d.row_len = m.dev.row_len;
    d.err = g_err;
    d.safe = g_safe;
    d.frame_bytes = p.frame_bytes;
    d.block_bytes = m.block_bytes;
    d.slots_div = fastdiv_make((uint32_t)m.slots);
    d.max_block_id = (uint32_t)(p.n_frames * m.slots);
    d.Hq = m.Hq; d.Hkv = m.Hkv; d.g = m.g; d.D = m.D; d.dtype = m.dtype;
}

int kv_read(int model, int seq, int tok_begin, int n_tok, void *k_out, void *v_out, float *k_scale_out,
            float *v_scale_out) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (seq < 0 || seq >= m->dev.max_seqs || tok_begin < 0 || n_tok < 0) return PKV_E_ARG;
    if (n_tok == 0) return 0;
    if (!k_out || !v_out) return PKV_E_ARG;
    if (m->dtype == PKV_E4M3 && (!k_scale_out || !v_scale_out)) return PKV_E_ARG;
    Pool &p = g_pools[m->pool];
    if (m->stale) {
        int rcs = reconcile_pool(m->pool);
        if (rcs) return rcs;
    }
    if (((int64_t)tok_begin + n_tok + p.T - 1) / p.T > m->row_len[seq]) return PKV_E_RANGE;
    AttnDesc d{};
    fill_addressing(d, *m);
    HIP_TRY(pkv_launch_kv_read(d, seq, tok_begin, n_tok, k_out, v_out, k_scale_out, v_scale_out, g_stream));
    return n_tok;
}

int kv_append_chunk(int model, int batch, const void *k_new, const void *v_new, const int32_t *q_lens,
                    const int32_t *ctx_lens) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (batch < 0 || batch > m->dev.max_seqs) return PKV_E_RANGE;
    if (batch == 0) return 0;
    if (!k_new || !v_new || !q_lens || !ctx_lens) return PKV_E_ARG;
    // one entry per (sequence, j-th page its chunk may touch): a chunk of n tokens that starts
    // anywhere in a page touches at most ceil(n / T) + 1 pages
    Pool &p = g_pools[m->pool];
    std::vector<int4> rows;
    int64_t first = 0;
    for (int s = 0; s < batch; ++s) {
        if (q_lens[s] < 0) return PKV_E_ARG;
        if (q_lens[s] > 0)
            for (int j = 0; j < (q_lens[s] + p.T - 1) / p.T + 1; ++j)
                rows.push_back(make_int4((int)first, q_lens[s], s, j));
        first += q_lens[s];
        if (first > (int64_t)1 << 24) return PKV_E_RANGE;
    }
    if (first == 0) return 0;
    if (rows.size() > m->vmap_cap) {
        HIP_TRY(hipStreamSynchronize(g_stream));
        (void)hipFree(m->vmap);
        m->vmap = nullptr;
        m->vmap_cap = 0;
        HIP_TRY(hipMalloc((void **)&m->vmap, rows.size() * 2 * sizeof(int4)));
        m->vmap_cap = rows.size() * 2;
    }
    // pageable source: the copy has read `rows` when the call returns, and runs in stream order
    HIP_TRY(hipMemcpyAsync(m->vmap, rows.data(), rows.size() * sizeof(int4), hipMemcpyHostToDevice, g_stream));
    AttnDesc d{};
    fill_addressing(d, *m);
    d.batch = (int)rows.size();
    d.ctx_lens = ctx_lens;
    d.vmap = m->vmap;
    HIP_TRY(pkv_launch_kv_append(d, k_new, v_new, g_stream));
    return (int)first;
}

int kv_append(int model, int batch, const void *k_new, const void *v_new, const int32_t *ctx_lens) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (batch < 0 || batch > m->dev.max_seqs) return PKV_E_RANGE;
    if (batch == 0) return 0;
    if (!k_new || !v_new || !ctx_lens) return PKV_E_ARG;
    AttnDesc d{};
    fill_addressing(d, *m);
    d.batch = batch;
    d.ctx_lens = ctx_lens;
    HIP_TRY(pkv_launch_kv_append(d, k_new, v_new, g_stream));
    return batch;
}

/* -------------------------------------------------------- decode attention */

int model_set_batch(int model, int batch, int row_stride) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (batch < 0 || row_stride < 0) return PKV_E_ARG;
    m->batch = batch;
    m->row_stride = row_stride;
    return PKV_OK;
}

int decode_attention_ex(int model, int batch, const void *q, const int32_t *block_table, int row_stride,
                        const int32_t *ctx_lens, float *out) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (batch < 0) return PKV_E_ARG;
    if (batch == 0) return PKV_OK;
    if (!q || !ctx_lens || !out) return PKV_E_ARG;
    if (((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return PKV_E_ARG;
    if (block_table) {
        if (row_stride <= 0) return PKV_E_ARG;
        // An elastic pool backs a frame with memory only while a model owns it, and the kernels cannot
        // tell whether an id of a caller's table points into such a frame: only the library's own table
        // (whose rows end where the model's live blocks end) is served there.
        if (g_pools[m->pool].elastic) {
            snprintf(g_errbuf, sizeof g_errbuf, "decode_attention: a caller's block table is not served on an elastic pool");
            return PKV_E_UNSUPPORTED;
        }
    } else if (batch > m->dev.max_seqs) {
        return PKV_E_RANGE;
    }
    AttnGroup grp;
    grp.n = 1;
    LaunchLoad load;
    load.add(*m, block_table == nullptr, batch, row_stride);
    plan_launch(load);
    int rc = fill_desc(grp.m[0], *m, batch, q, block_table, row_stride, ctx_lens, out, 1.0);
    if (rc) return rc;

    return launch_attention(grp);
}

int decode_attention_static(int model, int batch, const void *q, const int32_t *block_table, int row_stride,
                            const int32_t *ctx_lens, float *out) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (batch < 0) return PKV_E_ARG;
    if (batch == 0) return PKV_OK;
    if (!q || !ctx_lens || !out) return PKV_E_ARG;
    if (((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return PKV_E_ARG;
    if (block_table) {
        if (row_stride <= 0) return PKV_E_ARG;
        if (g_pools[m->pool].elastic) return PKV_E_UNSUPPORTED;
    } else if (batch > m->dev.max_seqs) {
        return PKV_E_RANGE;
    }
    const size_t n_cnt = (size_t)batch * m->Hkv;
    if (n_cnt > PKV_STATIC_COUNTERS) {
        snprintf(g_errbuf, sizeof g_errbuf, "decode_attention_static: batch * kv_heads = %zu exceeds the %d arrival counters of the scratch array",
                 n_cnt, PKV_STATIC_COUNTERS);
        return PKV_E_RANGE;
    }
    void *scratch_ptr = nullptr;
    HIP_TRY(pkv_static_scratch(&scratch_ptr));
    AttnGroup grp;
    grp.n = 1;
    g_deep_now = false;                   // the ordinary kernel form, every cache type
    g_plan_items = g_items > 0 ? g_items : kDefaultItems;
    AttnDesc &d = grp.m[0];
    fill_desc_core(d, *m, batch, q, block_table, row_stride, ctx_lens, out, 1.0);
    // the partials of the work items must fit what is left of the array behind the counters: fewer,
    // longer shares otherwise (any number of items gives the same result up to rounding)
    const size_t cnt_bytes = (size_t)PKV_STATIC_COUNTERS * sizeof(uint32_t);
    const size_t per_item = ws_floats_for(*m, 1, d.cols) * sizeof(float);
    const size_t fit = (PKV_STATIC_SCRATCH_BYTES - cnt_bytes) / per_item;
    if (fit < 1) return PKV_E_RANGE;
    if ((size_t)d.n_items > fit) {
        d.n_items = (int)fit;
        if (d.n_items >= 8) d.n_items &= ~7;
        d.weighted = d.n_items % 8 == 0 ? 1 : 0;
    }
    d.cnt = (uint32_t *)scratch_ptr;
    d.ws = (float *)((uint8_t *)scratch_ptr + cnt_bytes);
    fill_tune(grp.tune, false);
    HIP_TRY(pkv_launch_attention_static(grp, d.cnt, n_cnt, g_stream));
    return PKV_OK;
}

int prefill_attention(int model, int batch, const void *q, const int32_t *q_lens, const int32_t *ctx_lens, float *out) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (batch < 0 || batch > m->dev.max_seqs) return PKV_E_RANGE;
    if (batch == 0) return PKV_OK;
    if (!q || !q_lens || !ctx_lens || !out) return PKV_E_ARG;
    if (((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return PKV_E_ARG;
    // A wave takes as many consecutive query tokens as fit the 16 MFMA columns with the g heads of a
    // kv head; a work-group takes PKV_PREFILL_TILES such tiles and shares the K and V it fetches.
    const int tile = 16 / m->g > 0 ? 16 / m->g : 1;
    const int group = PKV_PREFILL_TILES * tile;
    std::vector<int4> rows;
    int64_t first = 0, n_groups = 0;
    for (int s = 0; s < batch; ++s) {
        if (q_lens[s] < 0) return PKV_E_ARG;
        n_groups += (q_lens[s] + group - 1) / group;
        first += q_lens[s];
        if (first > (int64_t)1 << 24) return PKV_E_RANGE;
    }
    if (n_groups == 0) return PKV_OK;
    // Few groups in front of long contexts would leave most of the chip idle: then every group comes
    // as several work-groups, each with a part of the context of at least kMinSplitPairs page pairs
    // (as far as the host can tell: it knows the blocks a row holds, not its context length).
    constexpr int kFillWorkGroups = 1024, kMinSplitPairs = 8, kMaxSplit = 64;
    const int64_t plain = n_groups * m->Hkv;
    const int want_split = plain >= kFillWorkGroups ? 1 : (int)((kFillWorkGroups + plain - 1) / plain);
    bool any_split = false;
    first = 0;
    for (int s = 0; s < batch; ++s) {
        const int est_pairs = (m->row_len[s] + 1) / 2;
        int n_split = want_split;
        if (n_split > est_pairs / kMinSplitPairs) n_split = est_pairs / kMinSplitPairs;
        if (n_split > kMaxSplit) n_split = kMaxSplit;
        if (n_split < 2) n_split = 0;
        // longest groups of a sequence first: they take the most pages
        for (int t0 = ((q_lens[s] - 1) / group) * group; q_lens[s] > 0 && t0 >= 0; t0 -= group) {
            const int n = q_lens[s] - t0 < group ? q_lens[s] - t0 : group;
            if (n_split == 0) rows.push_back(make_int4(s, (int)(first + t0), q_lens[s] - (t0 + n), n));
            for (int k = 0; k < n_split; ++k)
                rows.push_back(make_int4(s, (int)(first + t0), q_lens[s] - (t0 + n), n | (k << 8) | (n_split << 20)));
            any_split |= n_split > 0;
        }
        first += q_lens[s];
    }
    if (rows.size() > m->vmap_cap) {
        HIP_TRY(hipStreamSynchronize(g_stream));
        (void)hipFree(m->vmap);
        m->vmap = nullptr;
        m->vmap_cap = 0;
        HIP_TRY(hipMalloc((void **)&m->vmap, rows.size() * 2 * sizeof(int4)));
        m->vmap_cap = rows.size() * 2;
    }
    // pageable source: the copy has read `rows` when the call returns, and runs in stream order
    HIP_TRY(hipMemcpyAsync(m->vmap, rows.data(), rows.size() * sizeof(int4), hipMemcpyHostToDevice, g_stream));
    AttnDesc d{};
    fill_addressing(d, *m);
    d.q = (const uint16_t *)q;
    d.ctx_lens = ctx_lens;
    d.out = out;
    d.batch = batch;
    d.vmap = m->vmap;
    d.cols = tile * m->g;
    d.scale_log2 = (float)(1.4426950408889634 / sqrt((double)m->D));
    if (any_split) {
        const size_t need = rows.size() * m->Hkv * (PKV_PREFILL_TILES * 16) * (size_t)(m->D + 4);
        if (need > m->pf_ws_floats) {
            HIP_TRY(hipStreamSynchronize(g_stream));
            (void)hipFree(m->pf_ws);
            m->pf_ws = nullptr;
            m->pf_ws_floats = 0;
            HIP_TRY(hipMalloc((void **)&m->pf_ws, need * sizeof(float)));
            m->pf_ws_floats = need;
        }
        d.ws = m->pf_ws;
    }
    HIP_TRY(pkv_launch_prefill(d, (int)rows.size(), any_split, g_stream));
    return PKV_OK;
}

int decode_attention(int model, const void *q, const int32_t *block_table, const int32_t *ctx_lens, float *out) {
    Model *m = get_model(model);
    if (!m) return PKV_E_HANDLE;
    if (m->batch <= 0) return PKV_E_ARG;   // model_set_batch first
    return decode_attention_ex(model, m->batch, q, block_table, m->row_stride, ctx_lens, out);
}

int decode_attention_multi(int n_models, const int *models, const int *batches, const void *const *q,
                           const int32_t *const *ctx_lens, float *const *out) {
    if (n_models < 0 || n_models > PKV_MAX_GROUP) return PKV_E_ARG;
    if (n_models == 0) return PKV_OK;
    if (!models || !batches || !q || !ctx_lens || !out) return PKV_E_ARG;
    AttnGroup grp;
    grp.n = 0;
    int items = 0, pool = -1;
    double total_bytes = 0.0;
    LaunchLoad load;
    for (int i = 0; i < n_models; ++i) {
        Model *m = get_model(models[i]);
        if (!m) return PKV_E_HANDLE;
        for (int j = 0; j < i; ++j)
            if (models[j] == models[i]) return PKV_E_ARG;   // one partials buffer per model
        if (pool < 0) pool = m->pool;
        if (m->pool != pool) return PKV_E_ARG;
        if (batches[i] < 0 || batches[i] > m->dev.max_seqs) return PKV_E_RANGE;
        if (batches[i] == 0) continue;
        if (!q[i] || !ctx_lens[i] || !out[i]) return PKV_E_ARG;
        if (((uintptr_t)q[i] & 15) || ((uintptr_t)out[i] & 15)) return PKV_E_ARG;
        load.add(*m, true, batches[i], 0);
    }
    plan_launch(load);
    for (int i = 0; i < n_models; ++i)              // (the cost of a page depends on the form)
        if (batches[i] > 0) total_bytes += est_bytes(*get_model(models[i]), true, batches[i], 0) + 1.0;
    for (int i = 0; i < n_models; ++i) {
        if (batches[i] == 0) continue;
        Model *m = get_model(models[i]);
        AttnDesc &d = grp.m[grp.n];
        const double frac = (est_bytes(*m, true, batches[i], 0) + 1.0) / total_bytes;
        int rc = fill_desc(d, *m, batches[i], q[i], nullptr, 0, ctx_lens[i], out[i], frac);
        if (rc) return rc;
        d.item_begin = items;
        if (items % 8 != 0) d.weighted = 0;          // its items would not line up with the XCDs
        items += d.n_items;
        grp.n++;
    }
    if (grp.n == 0) return PKV_OK;
    return launch_attention(grp);
}

/* ------------------------------------------------------------ observation */

long pool_export_state(int pool, void *host_buf, size_t cap) {
    Pool *p = get_pool(pool);
    if (!p) return PKV_E_HANDLE;
    HIP_TRY(hipStreamSynchronize(g_stream));
    const int64_t nf = p->n_frames;
    std::vector<int32_t> img;
    int64_t n_free = 0;
    HIP_TRY(hipMemcpy(&n_free, p->dev.n_free, sizeof n_free, hipMemcpyDeviceToHost));
    std::vector<uint32_t> stack(nf);
    std::vector<int32_t> owner(nf);
    HIP_TRY(hipMemcpy(stack.data(), p->dev.free_stack, sizeof(uint32_t) * nf, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(owner.data(), p->dev.owner, sizeof(int32_t) * nf, hipMemcpyDeviceToHost));
    img.push_back(0x53564B50);
    img.push_back(1);
    img.push_back((int32_t)nf);
    img.push_back(p->T);
    img.push_back((int32_t)n_free);
    for (int64_t i = 0; i < n_free; ++i) img.push_back((int32_t)stack[i]);
    img.insert(img.end(), owner.begin(), owner.end());
    int n_models = 0;
    for (int id = 0; id < PKV_MAX_MODELS; ++id)
        if (g_models[id].live && g_models[id].pool == pool) n_models++;
    img.push_back(n_models);
    for (int id = 0; id < PKV_MAX_MODELS; ++id) {
        Model &m = g_models[id];
        if (!m.live || m.pool != pool) continue;
        int64_t cnt[2];
        HIP_TRY(hipMemcpy(cnt, m.dev.counters, sizeof cnt, hipMemcpyDeviceToHost));
        const int64_t owned = cnt[0];
        std::vector<uint32_t> frames(owned), bits((size_t)owned * m.dev.wpf);
        if (owned) {
            HIP_TRY(hipMemcpy(frames.data(), m.dev.frames, sizeof(uint32_t) * owned, hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(bits.data(), m.dev.bits, sizeof(uint32_t) * bits.size(), hipMemcpyDeviceToHost));
        }
        img.push_back(id); img.push_back(m.Hq); img.push_back(m.Hkv); img.push_back(m.D); img.push_back(m.dtype);
        img.push_back(m.slots); img.push_back((int32_t)owned);
        for (int64_t i = 0; i < owned; ++i) img.push_back((int32_t)frames[i]);
        const int64_t nbits = owned * m.slots;
        img.push_back((int32_t)nbits);
        std::vector<uint32_t> packed((size_t)((nbits + 31) / 32), 0u);
        for (int64_t i = 0; i < owned; ++i)          // per-frame words -> one contiguous bit string
            for (int s = 0; s < m.slots; ++s)
                if (bits[(size_t)i * m.dev.wpf + (s >> 5)] >> (s & 31) & 1u) {
                    const int64_t j = i * m.slots + s;
                    packed[(size_t)(j >> 5)] |= 1u << (j & 31);
                }
        for (uint32_t w : packed) img.push_back((int32_t)w);
        img.push_back(m.dev.max_seqs);
        std::vector<int32_t> len(m.dev.max_seqs);
        HIP_TRY(hipMemcpy(len.data(), m.dev.row_len, sizeof(int32_t) * len.size(), hipMemcpyDeviceToHost));
        int n_rows = 0;
        for (int32_t l : len) n_rows += l > 0;
        img.push_back(n_rows);
        std::vector<int32_t> row(m.dev.max_blocks);
        for (int s = 0; s < m.dev.max_seqs; ++s) {
            if (len[s] == 0) continue;
            HIP_TRY(hipMemcpy(row.data(), m.dev.rows + (size_t)s * m.dev.max_blocks, sizeof(int32_t) * len[s],
                              hipMemcpyDeviceToHost));
            img.push_back(s);
            img.push_back(len[s]);
            img.insert(img.end(), row.begin(), row.begin() + len[s]);
        }
    }
    const size_t need = img.size() * sizeof(int32_t);
    if (host_buf && cap >= need) memcpy(host_buf, img.data(), need);
    return (long)need;
}

int pool_stats(int pool, pkv_stats *out) {
    Pool *p = get_pool(pool);
    if (!p) return PKV_E_HANDLE;
    if (!out) return PKV_E_ARG;
    memset(out, 0, sizeof *out);
    HIP_TRY(hipStreamSynchronize(g_stream));
    int64_t n_free = 0;
    HIP_TRY(hipMemcpy(&n_free, p->dev.n_free, sizeof n_free, hipMemcpyDeviceToHost));
    out->n_frames = p->n_frames;
    out->n_free = n_free;
    for (int id = 0; id < PKV_MAX_MODELS; ++id) {
        Model &m = g_models[id];
        if (!m.live || m.pool != pool) continue;
        int64_t cnt[2];
        HIP_TRY(hipMemcpy(cnt, m.dev.counters, sizeof cnt, hipMemcpyDeviceToHost));
        out->owned[id] = cnt[0];
        out->used_blocks[id] = cnt[0] * m.slots - cnt[1];
    }
    out->mapped_bytes = p->n_frames * (int64_t)p->frame_bytes;
    if (p->elastic) {
        std::lock_guard<std::mutex> g(p->el->mu);
        out->mapped_bytes = p->el->mapped_frames * (int64_t)p->frame_bytes;
        out->idle_frames = p->el->mapped_free;
    }
    return PKV_OK;
}

}  // extern "C"
