// Host side of the C ABI declared in include/het_cache.h: argument checks, device memory
// owned by the cache, and the kernel sequence of each call.  No step of the method runs on the
// host; the host only decides launch shapes from sizes it already knows (n, max_batch_ids,
// capacity) and never waits for the device inside het_lookup / het_update.
#include "../../include/het_cache.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "cache_kernels.hpp"
#include "pattern_kernels.hpp"

using namespace het;

// Kernels of the path, as named in profiles and by het_profile_kernel_name.
enum KernelId {
    K_SORT_STAGE, K_PROBE, K_POOLED_INDEX, K_FILL_GATHER, K_APPLY, K_TRIM_STAGE,
    K_TRIM_EVICT, K_DEFERRED_PUSH, K_LINK, K_FLUSH, K_MISC, K_NUM
};
static const char *const kKernelNames[K_NUM] = {
    "sort_stage_kernel", "probe_kernel", "pooled_index_kernel", "fill_gather_kernel",
    "apply_kernel", "trim_stage_kernel", "trim_evict_kernel", "deferred_push_kernel", "link_kernel", "flush_kernel", "misc"};

struct ProfSpan { int id; hipEvent_t start, stop; };

constexpr int SORT_SETS = 4;
constexpr uint32_t FILL_MAX_BLOCKS = 1024;     // workgroups that fetch missed rows (more only queue up ahead of the gather's)

// A batch announced by het_prefetch: its ids, the buffer set its sort uses and how far the sort has come.
struct Announced {
    const int64_t *ids = nullptr;
    uint32_t n = 0;
    int set = 0;
    int next_stage = 0;              // stages [0, next_stage) are enqueued; 2 * passes stages in all
};

struct het_cache {
    // creation parameters
    int64_t capacity = 0, s = 0;
    int32_t dim = 0, policy = 0;
    // configuration
    bool configured = false, attached = false;
    bool many = false;               // one of several workers over one global table (het_cache_set_many_writers)
    uint32_t lfu_cap = 16;           // HET_POLICY_LFU_LIGHT: where the use counter stops
    int64_t max_ids = 0;
    int32_t optimizer = 0;
    float eps = 0.f;
    hipStream_t stream = nullptr;
    int location = 0;
    // device state
    CacheView cv{};
    Workspace ws{};
    ApplyBorders bd{};
    TrimPlan tp{};
    // Four sets of sort buffers: the order of the current batch (kept for its update) and up to
    // three batches announced ahead by het_prefetch, whose sorts are carried by the kernels of the
    // calls in between (a sort is more stages long than a lookup and an update have kernels, so
    // in steady state two announced batches are being sorted and a third stands ready).
    uint32_t *keys[SORT_SETS][2] = {}, *idx[SORT_SETS][2] = {};
    uint32_t *sort_hist[SORT_SETS] = {};
    int sort_set = 0;                // the set that holds the current batch's order
    Announced ann[SORT_SETS - 1];    // announced batches, oldest first
    int n_ann = 0;
    TrimPlan sel_tp{};               // the select plan of the rows now cached (fixed at the lookup)
    int sel_next = 1;                // first stage of that select which the lookup's kernels did not carry
    int h0_bits = 0;                 // iteration-count width the kept first-pass histogram was counted for (0: not counted yet)
    bool last_trim_skipped = false;  // the last update had nothing to trim: its evicted-id list is empty
    int cslot = 0;                   // which of the two per-call counter blocks the current call uses
    uint32_t *inv = nullptr;
    uint32_t *tile_free[2] = {nullptr, nullptr};   // free slots per tile, left by a trim; trims alternate between the two
    int tf_last = 0;                 // the one the last trim filled (initially: every slot free)
    uint32_t *ev_ids[2] = {nullptr, nullptr};      // evicted ids of the last two trims, alternating like tile_free
    uint32_t n_buckets = 0;
    int max_chunks_per_lane = 1;     // row chunks one lane handles in the apply kernel
    std::vector<void *> owned;       // every device allocation, for destroy
    char *arena = nullptr;           // one allocation that holds all the small arrays side by side (see dev_alloc)
    size_t arena_used = 0;
    // host-backed table: write-back of the last trim's victims still to be enqueued
    bool push_pending = false;
    int push_buf = 0;
    uint32_t push_seq = 0, trim_seq = 0;
    // host-backed table: the stream beside the main one on which rows of the coming batch are fetched
    // ahead and staged rows are written back while the update runs (Section 4.1, 4.2)
    hipStream_t side = nullptr;
    hipEvent_t ev_main = nullptr, ev_link = nullptr;
    bool link_outstanding = false;   // a kernel on that stream has not been waited for yet
    uint32_t pf_serial = 0;
    int pf_slot_next = 0;            // which of the two list counters the next list uses
    struct { bool ready = false; const int64_t *ids = nullptr; uint32_t n = 0, tag = 0; } pf;   // rows fetched ahead, and for which lookup
    // host-side bookkeeping
    uint64_t t_host = 0;             // non-empty lookups so far (equals the device's t)
    bool overflow_pending = false;   // a lookup ran and no trim since
    uint32_t last_lookup_n = 0;
    const int64_t *order_ids = nullptr;   // ids the current sorted order was built from (by a lookup)
    uint32_t order_n = 0;
    bool order_valid = false;
    // optional per-kernel timing (het_profile_begin / het_profile_end)
    bool profiling = false;
    KernelTrace trace[2]{};          // het_profile_trace: the update's kernel, the lookup's second kernel
    // The last lookup left the fetch of its missed keys' rows to the update that reuses its order (table in
    // HBM, one worker): that update reads them from the global table.  Any other call that needs the rows
    // in their slots fetches them first (settle_fetch).
    bool fetch_owed = false;
    uint32_t owed_n = 0, owed_t = 0;
    std::vector<ProfSpan> spans;
};

namespace {

// With HET_DEBUG set in the environment, a failing HIP call is named on stderr.
void report(const char *what, hipError_t e)
{
    if (std::getenv("HET_DEBUG")) std::fprintf(stderr, "[het_cache] %s: %s\n", what, hipGetErrorString(e));
}

#define HIP_TRY(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) { report(#expr, e_); return HET_EHIP; } \
    } while (0)

// Frees the device allocations made after the first `keep`, and what was taken from the arena after
// `arena_mark` (a call that fails midway leaves nothing behind).
void free_owned_from(het_cache *c, size_t keep, size_t arena_mark)
{
    while (c->owned.size() > keep) {
        if (c->owned.back() == c->arena) { c->arena = nullptr; c->arena_used = 0; }
        (void)hipFree(c->owned.back());
        c->owned.pop_back();
    }
    if (c->arena) c->arena_used = arena_mark;
}

constexpr size_t ARENA_BYTES = (size_t)128 << 20, ARENA_ITEM_MAX = 8u << 20;

// Arrays of up to 8 MB lie side by side in one allocation of 128 MB; larger ones, and whatever does
// not fit, get their own.  With an allocation per array the probe kernel's time on config 2 depended
// on how many arrays had been allocated before (13.0 or 14.5 us: two more small arrays were enough);
// side by side it does not.
template <typename T>
int dev_alloc(het_cache *c, T **p, size_t count)
{
    const size_t bytes = std::max<size_t>(count, 1) * sizeof(T);
    if (ARENA_BYTES && bytes <= ARENA_ITEM_MAX) {
        if (!c->arena) {
            void *a = nullptr;
            if (hipMalloc(&a, ARENA_BYTES) == hipSuccess) { c->arena = static_cast<char *>(a); c->arena_used = 0; c->owned.push_back(a); }
            else (void)hipGetLastError();
        }
        const size_t at = (c->arena_used + 255) / 256 * 256;
        if (c->arena && at + bytes <= ARENA_BYTES) {
            *p = reinterpret_cast<T *>(c->arena + at);
            c->arena_used = at + bytes;
            return HET_OK;
        }
    }
    void *q = nullptr;
    const hipError_t e = hipMalloc(&q, bytes);
    if (e != hipSuccess) { report("hipMalloc", e); return HET_ENOMEM; }
    c->owned.push_back(q);
    *p = static_cast<T *>(q);
    return HET_OK;
}

inline uint32_t cdiv(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

inline int bit_width(uint64_t v)
{
    int b = 0;
    while (v) { ++b; v >>= 1; }
    return b;
}

inline uint32_t pow2_at_least(uint64_t v)
{
    uint64_t p = 1;
    while (p < v) p <<= 1;
    return (uint32_t)p;
}

int status_from_bits(uint32_t bits)
{
    if (bits & ERRBIT_INTERNAL) return HET_EHIP;
    if (bits & ERRBIT_RANGE) return HET_ERANGE;
    if (bits & ERRBIT_STATE) return HET_ESTATE;
    return HET_OK;
}

// While profiling, every launch is bracketed by a pair of events on the cache's stream.
struct LaunchScope {
    het_cache *c;
    ProfSpan sp{};
    bool on;
    hipStream_t st;
    LaunchScope(het_cache *cache, int id, hipStream_t stream) : c(cache), on(cache->profiling), st(stream)
    {
        if (!on) return;
        sp.id = id;
        // timing only: no system-scope fence, whose cache write-back would be billed to the kernels
        if (hipEventCreateWithFlags(&sp.start, hipEventDisableSystemFence) != hipSuccess ||
            hipEventCreateWithFlags(&sp.stop, hipEventDisableSystemFence) != hipSuccess) { on = false; return; }
        (void)hipEventRecord(sp.start, st);
    }
    ~LaunchScope()
    {
        if (!on) return;
        (void)hipEventRecord(sp.stop, st);
        c->spans.push_back(sp);
    }
};
#define LAUNCH_ON(cache, stream_, id, ...)         \
    do {                                           \
        LaunchScope scope_(cache, id, stream_);    \
        __VA_ARGS__;                               \
    } while (0)
#define LAUNCH(cache, id, ...) LAUNCH_ON(cache, (cache)->stream, id, __VA_ARGS__)

int launch_ok()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { report("kernel launch", e); return HET_EHIP; }
    return HET_OK;
}

// Groups of `lanes` threads work on one row; how many 256-thread blocks for `items` rows.
uint32_t row_grid(const RowGeom &g, uint64_t items)
{
    const uint32_t per_block = 256u / (uint32_t)g.lanes;
    return std::max(1u, std::min(cdiv(items, per_block), 256u * 8u));      // at most 8 workgroups per CU
}

SortPlan make_sort_plan(const het_cache *c, uint32_t n, int set)
{
    SortPlan sp{};
    sp.n = n;
    sp.vocab = c->cv.vocab;
    const int bits = bit_width(sp.vocab);               // the key `vocab` itself marks a bad id
    sp.passes = std::max(1, (bits + SORT_MAX_BITS - 1) / SORT_MAX_BITS);
    sp.width = std::max(SORT_MIN_BITS, (bits + sp.passes - 1) / sp.passes);
    sp.ntiles = cdiv(n, SORT_TILE);
    sp.hist = c->sort_hist[set];
    return sp;
}

int sort_stages(const het_cache *c) { return 2 * make_sort_plan(c, 1, 0).passes; }
int sort_result_buffer(const het_cache *c) { return (make_sort_plan(c, 1, 0).passes - 1) & 1; }

// Stage `stage` of the sort of ids[n] into buffer set `set`.  Pass p writes buffer p & 1 of the
// set and reads the other one; stage 0 leaves the ids, converted to keys, where pass 0 reads.
SortStage make_stage(const het_cache *c, const int64_t *ids, uint32_t n, int set, int stage)
{
    SortStage s{};
    s.sp = make_sort_plan(c, n, set);
    const int pass = stage >> 1, out = pass & 1, in = 1 - out;
    s.ids = ids;
    s.keys_in = c->keys[set][in]; s.idx_in = c->idx[set][in];
    s.keys_out = stage == 0 ? c->keys[set][in] : c->keys[set][out];
    s.idx_out = c->idx[set][out];
    s.stage = stage;
    s.blocks = s.sp.ntiles;
    return s;
}

SortStage no_stage()
{
    SortStage s{};
    s.stage = -1;
    return s;
}

// Begins a call that touches the cache: per-call counters go to the other counter block.
void begin_call(het_cache *c)
{
    c->cslot = 1 - c->cslot;
    c->cv.last = &c->cv.ds->call[c->cslot];
    c->cv.next_call = &c->cv.ds->call[1 - c->cslot];
}

// Stages [first_stage, end) of a sort as kernels of their own.
void sort_now(het_cache *c, const int64_t *ids, uint32_t n, int set, int first_stage)
{
    for (int st = first_stage; st < sort_stages(c); ++st) {
        const SortStage s = make_stage(c, ids, n, set, st);
        LAUNCH(c, K_SORT_STAGE, sort_stage_kernel<<<s.blocks, SORT_THREADS, sort_stage_lds_bytes(s.sp.width, s.stage), c->stream>>>(s));
    }
}

// The next stage of the oldest announced batch whose sort is not complete yet, for the kernel
// that is about to be launched to carry.
SortStage next_ride_of(het_cache *c, int a)
{
    Announced &an = c->ann[a];
    return make_stage(c, an.ids, an.n, an.set, an.next_stage++);
}

// What the kernel about to be launched carries: the next stage of the oldest announced batch whose
// sort is not complete yet and, since stages of one sort need a kernel boundary between them, the
// next stage of the batch announced after it.
struct Rides {
    SortStage a, b;
    uint32_t blocks() const { return a.blocks + b.blocks; }
    // 0: nothing, 1: histogram stages only, 2: a scatter stage among them
    int kind() const { return !blocks() ? 0 : (((a.blocks && (a.stage & 1)) || (b.blocks && (b.stage & 1))) ? 2 : 1); }
};

// LDS a kernel needs: its own roles' or, if larger, a carried stage's.
uint32_t lds_bytes(size_t own, const Rides &r)
{
    uint32_t need = (uint32_t)own;
    if (r.a.blocks) need = std::max(need, sort_stage_lds_bytes(r.a.sp.width, r.a.stage));
    if (r.b.blocks) need = std::max(need, sort_stage_lds_bytes(r.b.sp.width, r.b.stage));
    return need;
}

Rides next_rides(het_cache *c)
{
    Rides r{no_stage(), no_stage()};
    int got = 0;
    for (int a = 0; a < c->n_ann && got < 2; ++a) {
        if (c->ann[a].next_stage >= sort_stages(c)) continue;
        (got == 0 ? r.a : r.b) = next_ride_of(c, a);
        ++got;
    }
    return r;
}

void drop_oldest_announcement(het_cache *c)
{
    for (int a = 0; a + 1 < c->n_ann; ++a) c->ann[a] = c->ann[a + 1];
    c->n_ann -= 1;
}

void use_order(het_cache *c, int set)
{
    const int buf = sort_result_buffer(c);
    c->sort_set = set;
    c->ws.skey = c->keys[set][buf];
    c->ws.perm = c->idx[set][buf];
}

// The trim's select plan for the rows cached after the lookup that just ran: stages 0..passes-1
// are histogram passes, stage `passes` is the tie count.
TrimPlan make_trim_plan(const het_cache *c)
{
    TrimPlan tp = c->tp;
    tp.lfu = c->policy == HET_POLICY_LFU || c->policy == HET_POLICY_LFU_LIGHT;
    tp.bits = std::max(1, bit_width(c->t_host));
    tp.key_bits = tp.lfu ? 2 * tp.bits : tp.bits;
    tp.passes = (tp.key_bits + SEL_BITS - 1) / SEL_BITS;
    tp.sup_cnt = reinterpret_cast<uint4 *>(tp.hist + SEL_MAX_PASSES * SEL_BINS);
    return tp;
}

uint32_t stage_blocks(const het_cache *c, const TrimPlan &tp, int stage)
{
    if (stage < tp.passes) return std::min(cdiv(c->cv.n_slots, TRIM_TILE), 1024u);
    return cdiv(c->cv.n_slots, COUNT_SLOTS);
}

constexpr uint32_t STALE_BLOCKS = 128;     // fetch workgroups of a lookup that leaves the missed rows to the update: they refresh the stale rows
constexpr uint32_t PUSH_BLOCKS = 256;      // few workgroups keep the host link full; more only contend
constexpr uint32_t LINK_BLOCKS = 32;       // workgroups of the kernel that works the host link beside the update (half write back, half fetch ahead)

// Host-backed table: the main stream goes on only when the kernel on the stream beside it is done.
void wait_link(het_cache *c)
{
    if (!c->link_outstanding) return;
    (void)hipStreamWaitEvent(c->stream, c->ev_link, 0);
    c->link_outstanding = false;
}

// Host-backed table: enqueues the write-back a trim left staged, if nobody carried it yet.
void drain_pushes(het_cache *c)
{
    if (!c->push_pending) return;
    wait_link(c);                // (staged copies reach the table in the order they were staged)
    if (c->cv.geom.vec == 4) LAUNCH(c, K_DEFERRED_PUSH, deferred_push_kernel<4><<<PUSH_BLOCKS, 256, 0, c->stream>>>(c->cv, c->push_buf));
    else LAUNCH(c, K_DEFERRED_PUSH, deferred_push_kernel<1><<<PUSH_BLOCKS, 256, 0, c->stream>>>(c->cv, c->push_buf));
    c->push_pending = false;
}

// A lookup left the fetch of its missed keys' rows to the update that reuses its order, and that
// update is not what comes next: fetch them now (the lookup's lists are still in place: nothing
// has sorted, probed or trimmed since).
template <int VEC>
int settle_fetch_impl(het_cache *c)
{
    const uint32_t n = c->owed_n, ptiles = cdiv(n, PT_TILE);
    const uint32_t fill_blocks = std::min(cdiv(row_grid(c->cv.geom, n), (uint32_t)FILL_ROWS), FILL_MAX_BLOCKS);
    const TrimPlan none{};
    const SortStage no = no_stage();
    LAUNCH(c, K_FILL_GATHER, fill_gather_kernel<VEC, false, 0, false><<<fill_blocks, 256, sizeof(FillLds), c->stream>>>(
                                 c->cv, c->ws, n, c->owed_t, ptiles, fill_blocks, none, 0u, nullptr, nullptr, 0u, nullptr, no, no,
                                 0u, 0, 0u, 0, Ahead{}, KernelTrace{}, 2));
    c->fetch_owed = false;
    return launch_ok();
}
int settle_fetch(het_cache *c)
{
    if (!c->fetch_owed) return HET_OK;
    return c->cv.geom.vec == 4 ? settle_fetch_impl<4>(c) : settle_fetch_impl<1>(c);
}

// Evict(): the select stages from `first_stage` on (earlier ones rode along with the update's
// kernels), then the eviction itself.
template <int VEC>
int run_trim(het_cache *c, int first_stage)
{
    TrimPlan tp = c->sel_tp;
    drain_pushes(c);                                 // the staging buffers alternate: the one before last must be gone
    for (int st = first_stage; st <= tp.passes; ++st)
        LAUNCH(c, K_TRIM_STAGE, trim_stage_kernel<<<stage_blocks(c, tp, st), TRIM_THREADS, 0, c->stream>>>(c->cv, tp, st));
    const int fill = 1 - c->tf_last;                 // the idle array: cleared by the lookup in between
    tp.tile_free = c->tile_free[fill];
    tp.ev_slot = fill;
    tp.ev_ids = c->ev_ids[fill];
    tp.push_seq = ++c->trim_seq;
    if (c->trim_seq == 0x7FFFFFFFu) c->trim_seq = 0;        // 0 means "none", the top bit marks lists of keys fetched ahead; a wrap is harmless (see HostLink::pend)
    const Rides ride = next_rides(c);
    const uint32_t ev_blocks = cdiv(c->cv.n_slots, EV_SLOTS);
    // Rows of a kilobyte or more: the pushes run at the memory's limit, and a fourth workgroup per
    // compute unit only gets in the others' way (config 5: 107 us against 97).  Asking for more LDS
    // than a quarter of a compute unit's keeps it to three.  Not where the update pushes the rows it
    // fetches early: then few victims are left to copy, and the fourth workgroup pays (config 5:
    // 25.9 -> 23.5 us).
    const uint32_t lds_floor = c->cv.geom.lanes == 64 && VEC == 4 && !c->cv.early_cc ? 44u * 1024u : 0u;
    const uint32_t lds = std::max(lds_bytes(sizeof(EvictLds), ride), lds_floor);
    if (c->many)
        LAUNCH(c, K_TRIM_EVICT, trim_evict_kernel<VEC, true, true><<<ride.blocks() + ev_blocks + 1, TRIM_THREADS, lds, c->stream>>>(c->cv, tp, ride.a, ride.b));
    else if (ride.blocks())
        LAUNCH(c, K_TRIM_EVICT, trim_evict_kernel<VEC, true, false><<<ride.blocks() + ev_blocks + 1, TRIM_THREADS, lds, c->stream>>>(c->cv, tp, ride.a, ride.b));
    else
        LAUNCH(c, K_TRIM_EVICT, trim_evict_kernel<VEC, false, false><<<ev_blocks + 1, TRIM_THREADS, lds, c->stream>>>(c->cv, tp, ride.a, ride.b));
    c->tf_last = fill;
    if (c->location == HET_BACKING_PINNED_HOST) { c->push_pending = true; c->push_buf = fill; c->push_seq = tp.push_seq; }
    c->overflow_pending = false;
    c->last_trim_skipped = false;
    c->order_valid = false;          // slots recorded for the sorted order may be gone now
    return launch_ok();
}

template <int VEC>
int run_lookup(het_cache *c, const int64_t *ids, uint32_t n, const int64_t *offsets, uint32_t n_bags, float *out)
{
    begin_call(c);
    c->t_host += 1;
    int rc;
    if ((rc = settle_fetch(c)) != HET_OK) return rc;
    if (c->overflow_pending && (rc = run_trim<VEC>(c, c->sel_next)) != HET_OK) return rc;   // a Read that follows a Read
    // The sorted order: announced by het_prefetch and sorted inside the kernels launched since
    // (what is left of it runs now), or sorted here.  Announcements older than the one used are
    // void; with no match they all stand (a later lookup may still use them).
    int match = -1;
    for (int a = 0; a < c->n_ann && match < 0; ++a)
        if (c->ann[a].ids == ids && c->ann[a].n == n) match = a;
    if (match >= 0) {
        for (int a = 0; a < match; ++a) drop_oldest_announcement(c);
        const Announced an = c->ann[0];
        drop_oldest_announcement(c);
        sort_now(c, ids, n, an.set, an.next_stage);
        use_order(c, an.set);
    } else {
        sort_now(c, ids, n, c->sort_set, 0);             // over the previous batch's order: it is not needed any more
        use_order(c, c->sort_set);
    }
    const uint32_t t_now = (uint32_t)c->t_host;
    if (c->cv.direct) {
        // no cache: mark the runs, then gather straight from the global table
        LAUNCH(c, K_PROBE, direct_probe_kernel<true><<<cdiv(n, PT_TILE) * (match >= 0 ? 2u : 1u), PT_THREADS, 0, c->stream>>>(c->cv, c->ws, n, t_now, cdiv(n, PT_TILE), match >= 0 ? ids : nullptr,
                                                                                                                              offsets ? c->inv : nullptr));
        const Rides ride = next_rides(c);
        const uint32_t grid = ride.blocks() + row_grid(c->cv.geom, offsets ? n_bags : cdiv(n, GATHER_ROWS));
        const uint32_t lds = lds_bytes(std::max(sizeof(FillLds), sizeof(TrimLds)), ride);
        const TrimPlan none{};
#define GATHER_ONLY_T(POOLED, RIDE, TRACE)                                                                               \
    LAUNCH(c, K_FILL_GATHER, fill_gather_kernel<VEC, POOLED, RIDE, TRACE><<<grid, 256, lds, c->stream>>>(                   \
                                 c->cv, c->ws, n, t_now, 0u, 0u, none, 0u, out, offsets, n_bags, c->inv, ride.a, ride.b, 0u, 0, 0u, 0, Ahead{}, c->trace[1], 0))
#define GATHER_ONLY(POOLED, RIDE) do { if (c->trace[1].rec) GATHER_ONLY_T(POOLED, RIDE, true); else GATHER_ONLY_T(POOLED, RIDE, false); } while (0)
        const int kind = ride.kind();
        if (!offsets) { if (kind == 0) GATHER_ONLY(false, 0); else if (kind == 1) GATHER_ONLY(false, 1); else GATHER_ONLY(false, 2); }
        else { if (kind == 0) GATHER_ONLY(true, 0); else if (kind == 1) GATHER_ONLY(true, 1); else GATHER_ONLY(true, 2); }
#undef GATHER_ONLY
#undef GATHER_ONLY_T
        if ((rc = launch_ok()) != HET_OK) return rc;
        c->last_lookup_n = n;
        c->order_ids = ids; c->order_n = n; c->order_valid = true;
        return HET_OK;
    }
    const uint32_t ptiles = cdiv(n, PT_TILE), stiles = cdiv(c->cv.n_slots, PT_TILE);
    // The select plan of the trim that follows this lookup.  Its first pass's histogram is kept
    // between trims as long as the digit layout (the width of the iteration count) stays the same;
    // otherwise this lookup counts it afresh, beside its fetches.
    c->sel_tp = make_trim_plan(c);
    c->sel_tp.h0_kept = c->h0_bits == c->sel_tp.bits;
    c->h0_bits = c->sel_tp.bits;
    const TrimPlan &tp = c->sel_tp;
    const uint32_t kept_words = tp.h0_kept ? (uint32_t)SEL_BINS : 0u;
    LAUNCH(c, K_PROBE, probe_kernel<true><<<ptiles + (match >= 0 ? ptiles : 0u) + stiles, PT_THREADS, 0, c->stream>>>(
                           c->cv, c->ws, n, t_now, ptiles, c->tile_free[c->tf_last], c->tile_free[1 - c->tf_last], (uint32_t)(1 - c->tf_last),
                           c->tp.hist + kept_words, c->tp.zero_words - kept_words, tp, match >= 0 ? ids : nullptr,
                           c->side ? c->pf_slot_next : -1, offsets ? c->inv : nullptr));
    const int hist_pass = tp.h0_kept ? 1 : 0;                  // this pass of the select rides with the fetches
    // (the update has one kernel to carry a stage: with the first pass kept, a select of two passes
    // is over when that kernel ends: second pass here, tie count there)
    const uint32_t hist_blocks = hist_pass < tp.passes ? stage_blocks(c, tp, hist_pass) : 0u;
    c->sel_next = hist_blocks ? hist_pass + 1 : hist_pass;     // (a select of one pass whose histogram is kept: only the tie count is left)
        const uint32_t fill_blocks = std::min(cdiv(row_grid(c->cv.geom, n), (uint32_t)FILL_ROWS), FILL_MAX_BLOCKS);     // they come first: theirs is the longer chain
    const uint32_t lds_own = (uint32_t)std::max(sizeof(FillLds), sizeof(TrimLds));
#define FILL_GATHER_T(POOLED, RIDE, TRACE, GRID, FILLB, HISTB, PUSHB)                                                     \
    LAUNCH(c, K_FILL_GATHER, fill_gather_kernel<VEC, POOLED, RIDE, TRACE><<<GRID, 256, lds_bytes(lds_own, ride), c->stream>>>( \
                                 c->cv, c->ws, n, t_now, ptiles, FILLB, tp, HISTB, out, offsets, n_bags, c->inv, ride.a, ride.b, \
                                 PUSHB, c->push_buf, c->push_seq, hist_pass, ah, c->trace[1], fetch_mode))
#define FILL_GATHER(POOLED, RIDE, GRID, FILLB, HISTB, PUSHB)                                                              \
    do {                                                                                                                  \
        if (c->trace[1].rec) FILL_GATHER_T(POOLED, RIDE, true, GRID, FILLB, HISTB, PUSHB);                                \
        else FILL_GATHER_T(POOLED, RIDE, false, GRID, FILLB, HISTB, PUSHB);                                               \
    } while (0)
#define FILL_GATHER_ANY(GRID, FILLB, HISTB, PUSHB)                                                                        \
    do {                                                                                                                  \
        const int kind = ride.kind();                                                                                     \
        if (!offsets) {                                                                                                   \
            if (kind == 0) FILL_GATHER(false, 0, GRID, FILLB, HISTB, PUSHB);                                              \
            else if (kind == 1) FILL_GATHER(false, 1, GRID, FILLB, HISTB, PUSHB);                                         \
            else FILL_GATHER(false, 2, GRID, FILLB, HISTB, PUSHB);                                                        \
        } else {                                                                                                          \
            if (kind == 0) FILL_GATHER(true, 0, GRID, FILLB, HISTB, PUSHB);                                               \
            else if (kind == 1) FILL_GATHER(true, 1, GRID, FILLB, HISTB, PUSHB);                                          \
            else FILL_GATHER(true, 2, GRID, FILLB, HISTB, PUSHB);                                                         \
        }                                                                                                                 \
    } while (0)
    const uint32_t gather_blocks = row_grid(c->cv.geom, offsets ? n_bags : cdiv(n, GATHER_ROWS));
    Ahead ah{};
    int fetch_mode = 0;
    if (c->location == HET_BACKING_HBM && !c->many) {
        // one kernel: the gather reads a missed key's row from the global table, beside the fetch.
        // The missed keys' rows themselves are left to the update that is expected to follow (it reads
        // them from the global table and writes them to their slots with its step applied); the fetch
        // workgroups that remain refresh the stale rows.
        const Rides ride = next_rides(c);
        const bool owe = !c->cv.rowwise;
        fetch_mode = owe ? 1 : 0;
        const uint32_t fb = owe ? std::min(fill_blocks, STALE_BLOCKS) : fill_blocks;
        FILL_GATHER_ANY(ride.blocks() + fb + ptiles + hist_blocks + gather_blocks, fb, hist_blocks, 0u);
        if (owe) { c->fetch_owed = true; c->owed_n = n; c->owed_t = t_now; }
    } else {
        // Host-backed table: the fetches come over the host link, and the last trim's write-back
        // goes the other way in the same kernel; the gather follows and reads the cached copies.
        // Several workers: a row that is synchronised takes a new value (the server's row plus this
        // worker's push), which the gather must see, so it follows in a launch of its own too.
        // Host-backed table with a batch announced for the next lookup: the second kernel lists that
        // batch's keys that are not cached, and a kernel on the stream beside this one brings their rows
        // into HBM while the update runs, with the write-back going the other way beside them (so the
        // fetch kernel leaves the write-back to it); the next lookup's fetch kernel finds them there.
        const bool host = c->side != nullptr;
        Announced *next = host && c->n_ann > 0 ? &c->ann[0] : nullptr;
        if (host) {
            // rows fetched ahead for this lookup; and no refresh of this lookup may overtake an older staged copy
            wait_link(c);
            if (c->pf.ready && c->pf.ids == ids && c->pf.n == n) ah.use_tag = c->pf.tag;
            c->pf.ready = false;
        }
        const uint32_t push_blocks = c->push_pending && !next ? PUSH_BLOCKS : 0u;
        const uint32_t fetch_blocks = c->location == HET_BACKING_HBM ? fill_blocks : std::min(fill_blocks, PUSH_BLOCKS);
        {
            const Rides ride = next_rides(c);
            FILL_GATHER_ANY(ride.blocks() + push_blocks + fetch_blocks + ptiles + hist_blocks, fetch_blocks, hist_blocks, push_blocks);
        }
        if (push_blocks) c->push_pending = false;
        ah = Ahead{};
        if (next) {
            if (next->next_stage < sort_stages(c)) {         // what is left of its sort runs now
                sort_now(c, next->ids, next->n, next->set, next->next_stage);
                next->next_stage = sort_stages(c);
            }
            c->pf_serial = (c->pf_serial % 0x7FFFFFFFu) + 1;
            ah.skey = c->keys[next->set][sort_result_buffer(c)];
            ah.n = next->n;
            ah.blocks = cdiv(next->n, 256);
            ah.list_tag = 0x80000000u | c->pf_serial;
            ah.list_slot = c->pf_slot_next;
            ah.pending_seq = c->push_pending ? c->push_seq : 0u;
        }
        {
            const Rides ride = next_rides(c);
            FILL_GATHER_ANY(ride.blocks() + ah.blocks + gather_blocks, 0u, 0u, 0u);
        }
        if (next) {
            if ((rc = launch_ok()) != HET_OK) return rc;
            HIP_TRY(hipEventRecord(c->ev_main, c->stream));
            HIP_TRY(hipStreamWaitEvent(c->side, c->ev_main, 0));
            const int pbuf = c->push_pending ? c->push_buf : -1;
            // Few workgroups with several rows in flight each: a compute unit that waits for the host link
            // serves its other waves' memory requests behind those that wait, so every compute unit that
            // hosts a workgroup of this kernel is slow for the update's kernels meanwhile (measured: with
            // 512 workgroups the optimizer step took as long as the whole transfer).
            if (VEC == 4) LAUNCH_ON(c, c->side, K_LINK, link_kernel<4><<<LINK_BLOCKS, 256, 0, c->side>>>(c->cv, pbuf, ah.list_slot, c->push_buf, LINK_BLOCKS / 2));
            else LAUNCH_ON(c, c->side, K_LINK, link_kernel<1><<<LINK_BLOCKS, 256, 0, c->side>>>(c->cv, pbuf, ah.list_slot, c->push_buf, LINK_BLOCKS / 2));
            if ((rc = launch_ok()) != HET_OK) return rc;
            HIP_TRY(hipEventRecord(c->ev_link, c->side));
            c->link_outstanding = true;
            c->push_pending = false;
            c->pf.ready = true; c->pf.ids = next->ids; c->pf.n = next->n; c->pf.tag = ah.list_tag;
            c->pf_slot_next ^= 1;
        }
    }
#undef FILL_GATHER_ANY
#undef FILL_GATHER
#undef FILL_GATHER_T
    if ((rc = launch_ok()) != HET_OK) return rc;
    c->overflow_pending = true;
    c->last_lookup_n = n;
    c->order_ids = ids; c->order_n = n; c->order_valid = true;
    return HET_OK;
}

// The kernel of Write.  It carries one stage of the coming trim's select in extra workgroups (the
// stages before c->sel_next are done: the kept first pass, and what rode with the lookup's
// fetches): a histogram pass (policy fields only), or the tie count.  The count looks at the clocks
// the kernel is moving, which is sound only when the update is known to touch exactly the rows the
// last Read touched (it reuses that Read's order): see TrimPlan::dirty_stamp.
// `trim`: a trim follows.  Returns the first stage that is still to run.
template <int VEC, int MAXC, int TILE, bool EARLY>
int launch_apply_tile2(het_cache *c, bool verify, const int64_t *ids, uint32_t n, const float *grads, const uint32_t *grad_row, float lr,
                      bool trim)
{
    const uint32_t grid = cdiv(n, TILE);
    TrimPlan tp = c->sel_tp;
    int next = c->sel_next;
    int stage = -1;
    if (trim && next < tp.passes) stage = next++;
    else if (trim && next == tp.passes && verify && !c->cv.freq_cap) { stage = next++; tp.dirty_stamp = (uint32_t)c->t_host; }    // (light-weight LFU leaves some rows of the batch unstamped)
    const uint32_t extra = stage >= 0 ? stage_blocks(c, tp, stage) : 0u;
    const Rides ride = next_rides(c);
    const int fresh = verify && c->fetch_owed ? 1 : 0;          // (verify: this update reuses the lookup's order)
    if (fresh) c->fetch_owed = false;
    const uint32_t lds = lds_bytes(std::max(sizeof(TrimLds), sizeof(ApplyLds<VEC, TILE>)), ride);
    if (verify)
        LAUNCH(c, K_APPLY, apply_kernel<VEC, MAXC, true, TILE, EARLY><<<ride.blocks() + grid + extra + cdiv(n, VERIFY_TILE), AP_THREADS, lds, c->stream>>>(c->cv, c->ws, c->bd, ids, grads, grad_row, lr, c->eps, n, grid, tp, stage, ride.a, ride.b, c->trace[0], fresh));
    else
        LAUNCH(c, K_APPLY, apply_kernel<VEC, MAXC, false, TILE, EARLY><<<ride.blocks() + grid + extra, AP_THREADS, lds, c->stream>>>(c->cv, c->ws, c->bd, ids, grads, grad_row, lr, c->eps, n, grid, tp, stage, ride.a, ride.b, c->trace[0], fresh));
    return next;
}

// EARLY: the variant that also pushes the rows it fetches (CacheView::early_cc in use).
template <int VEC, int MAXC, int TILE>
int launch_apply_tile(het_cache *c, bool verify, const int64_t *ids, uint32_t n, const float *grads, const uint32_t *grad_row, float lr,
                      bool trim)
{
    if constexpr (VEC == 4)          // (only rows of whole 16-byte pieces push early)
        if (c->cv.early_cc) return launch_apply_tile2<VEC, MAXC, TILE, true>(c, verify, ids, n, grads, grad_row, lr, trim);
    return launch_apply_tile2<VEC, MAXC, TILE, false>(c, verify, ids, n, grads, grad_row, lr, trim);
}

template <int VEC, int MAXC>
int launch_apply(het_cache *c, bool verify, const int64_t *ids, uint32_t n, const float *grads, const uint32_t *grad_row, float lr,
                 bool trim)
{
    // rows of more than 128 floats (64 lanes to a row) have one row piece per lane or more; narrower ones exactly one
    if constexpr (MAXC == 1)
        if (ap_tile_for(c->cv.geom.lanes) == 64) return launch_apply_tile<VEC, MAXC, 64>(c, verify, ids, n, grads, grad_row, lr, trim);
    return launch_apply_tile<VEC, MAXC, 128>(c, verify, ids, n, grads, grad_row, lr, trim);
}

template <int VEC>
int run_update(het_cache *c, const int64_t *ids, uint32_t n, const int64_t *offsets, uint32_t n_bags,
               const float *grads, float lr)
{
    begin_call(c);
    int rc;
    // The ids of the preceding lookup, passed again: reuse its sorted order (the apply kernel
    // checks every id against it).  Anything else is sorted and probed afresh, into the current
    // set of sort buffers (announced batches use the other sets).
    const bool reuse = c->order_valid && ids == c->order_ids && n == c->order_n;
    if (!reuse) {
        if ((rc = settle_fetch(c)) != HET_OK) return rc;
        sort_now(c, ids, n, c->sort_set, 0);
        use_order(c, c->sort_set);
        if (c->cv.direct)
            LAUNCH(c, K_PROBE, direct_probe_kernel<false><<<cdiv(n, PT_TILE), PT_THREADS, 0, c->stream>>>(c->cv, c->ws, n, (uint32_t)c->t_host, cdiv(n, PT_TILE), nullptr));
        else
            LAUNCH(c, K_PROBE, probe_kernel<false><<<cdiv(n, PT_TILE), PT_THREADS, 0, c->stream>>>(
                                   c->cv, c->ws, n, (uint32_t)c->t_host, cdiv(n, PT_TILE), nullptr, nullptr, 0u, nullptr, 0u, TrimPlan{}, nullptr));
    }
    const uint32_t *grad_row = nullptr;
    if (offsets) {
        LAUNCH(c, K_POOLED_INDEX, pooled_index_kernel<<<std::min(cdiv(n, 256), 4096u), 256, 0, c->stream>>>(c->ws, n, offsets, n_bags));
        grad_row = c->ws.bag_of;
    }
    // Only a lookup leaves rows above capacity; an update that follows no lookup has nothing to trim.
    const bool trim = c->overflow_pending;
    int next_stage = 1;
    switch (c->max_chunks_per_lane) {
    case 1: next_stage = launch_apply<VEC, 1>(c, reuse, ids, n, grads, grad_row, lr, trim); break;
    case 2: next_stage = launch_apply<VEC, 2>(c, reuse, ids, n, grads, grad_row, lr, trim); break;
    case 4: next_stage = launch_apply<VEC, 4>(c, reuse, ids, n, grads, grad_row, lr, trim); break;
    default: next_stage = launch_apply<VEC, 16>(c, reuse, ids, n, grads, grad_row, lr, trim); break;
    }
    if ((rc = launch_ok()) != HET_OK) return rc;
    if (!trim) { c->last_trim_skipped = true; c->order_valid = false; return HET_OK; }
    return run_trim<VEC>(c, next_stage);
}

int sync_all(het_cache *c)
{
    drain_pushes(c);
    if (c->side) HIP_TRY(hipStreamSynchronize(c->side));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return HET_OK;
}

int sync_and_status(het_cache *c, DState *host_copy)
{
    int rc0 = sync_all(c);
    if (rc0) return rc0;
    DState h;
    HIP_TRY(hipMemcpy(&h, c->cv.ds, sizeof(DState), hipMemcpyDeviceToHost));
    if (host_copy) *host_copy = h;
    return status_from_bits(h.err);
}

void to_public(const Counters &in, het_counters *out)
{
    out->n = (int64_t)in.n; out->unique = (int64_t)in.unique; out->hit = (int64_t)in.hit;
    out->stale = (int64_t)in.stale; out->miss = (int64_t)in.miss; out->evicted = (int64_t)in.evicted;
    out->evicted_dirty = (int64_t)in.evicted_dirty; out->stale_dirty = (int64_t)in.stale_dirty;
    out->flushed = (int64_t)in.flushed;
}

bool ready(const het_cache *c) { return c && c->configured && c->attached; }

} // namespace

extern "C" {

int het_cache_create(het_cache **out, int64_t capacity, int32_t dim, int64_t s, int32_t policy)
{
    if (!out || capacity <= 0 || dim <= 0 || s < 0) return HET_EINVAL;
    if (policy != HET_POLICY_LRU && policy != HET_POLICY_LFU && policy != HET_POLICY_NONE && policy != HET_POLICY_LFU_LIGHT) return HET_EINVAL;
    if (capacity >= (1ll << 30) || dim > (1 << 20)) return HET_EINVAL;
    het_cache *c = new (std::nothrow) het_cache();
    if (!c) return HET_ENOMEM;
    c->capacity = capacity; c->dim = dim; c->s = s; c->policy = policy;
    *out = c;
    return HET_OK;
}

static int configure_impl(het_cache *c, int64_t max_batch_ids, int32_t optimizer, float eps, void *hip_stream)
{
    if (!c || c->configured || max_batch_ids <= 0 || max_batch_ids > (int64_t)MAX_PROBE_TILES * PT_TILE) return HET_EINVAL;
    if (optimizer != HET_OPT_SGD && optimizer != HET_OPT_ADAGRAD && optimizer != HET_OPT_ADAGRAD_ROWWISE) return HET_EINVAL;
    if (!(eps >= 0.f)) return HET_EINVAL;
    if (optimizer == HET_OPT_ADAGRAD_ROWWISE && c->many) return HET_EINVAL;
    c->max_ids = max_batch_ids; c->optimizer = optimizer; c->eps = eps;
    c->stream = static_cast<hipStream_t>(hip_stream);

    CacheView &cv = c->cv;
    const bool direct = c->policy == HET_POLICY_NONE;       // no cache: rows and accumulators are the global table's (set at attach)
    cv.direct = direct;
    const uint64_t P = direct ? 1 : (uint64_t)c->capacity + (uint64_t)max_batch_ids;
    cv.n_slots = (uint32_t)P; cv.capacity = (uint32_t)c->capacity; cv.max_ids = (uint32_t)max_batch_ids;
    cv.s = c->s; cv.adagrad = optimizer == HET_OPT_ADAGRAD; cv.rowwise = optimizer == HET_OPT_ADAGRAD_ROWWISE;
    RowGeom g;
    g.dim = c->dim; g.vec = (c->dim % 4 == 0) ? 4 : 1; g.chunks = c->dim / g.vec;
    g.lanes = (int)std::min<uint32_t>(64u, pow2_at_least((uint64_t)g.chunks));
    cv.geom = g;
    const int per_lane = (g.chunks + g.lanes - 1) / g.lanes;
    c->max_chunks_per_lane = per_lane <= 1 ? 1 : (per_lane <= 2 ? 2 : (per_lane <= 4 ? 4 : 16));
    if (per_lane > 16) return HET_EINVAL;               // rows wider than 64 lanes x 16 chunks
    if (cv.rowwise && per_lane > 1) return HET_EINVAL;  // row-wise Adagrad: the row group holds the whole row's gradient at once

    int rc = HET_OK;
    const size_t row_elems = (size_t)P * (size_t)c->dim;
    if (!direct && (rc = dev_alloc(c, &cv.rows, row_elems))) return rc;
    if (!direct && cv.adagrad && (rc = dev_alloc(c, &cv.acc, row_elems))) return rc;
    if (!direct && cv.rowwise && (rc = dev_alloc(c, &cv.acc, (size_t)P))) return rc;
    cv.many = c->many;
    // Early push where rows have 128 floats or more (measured: config 4 1.4 %, config 5 6 % faster; with
    // rows of 64 floats the update loses what the eviction gains).
    if (!direct && !c->many && !cv.rowwise && g.vec == 4 && g.lanes >= 32) {          // (dropped again at attach if the table is behind the host link)
        if ((rc = dev_alloc(c, &cv.early_cc, (size_t)P))) return rc;
        HIP_TRY(hipMemsetAsync(cv.early_cc, 0, (size_t)P * sizeof(uint32_t), c->stream));
    }
    cv.freq_cap = c->policy == HET_POLICY_LFU_LIGHT ? c->lfu_cap : 0u;
    if (c->many && (rc = dev_alloc(c, &cv.rows0, row_elems))) return rc;
    if (c->many && cv.adagrad && (rc = dev_alloc(c, &cv.acc0, row_elems))) return rc;
    if ((rc = dev_alloc(c, &cv.slot_key, P)) || (rc = dev_alloc(c, &cv.meta, P))) return rc;
    if ((rc = dev_alloc(c, &cv.free_list, (size_t)max_batch_ids)) || (rc = dev_alloc(c, &cv.was_free, P))) return rc;
    if ((rc = dev_alloc(c, &cv.ds, 1))) return rc;
    // hash table: at most a quarter of the entries are ever used
    c->n_buckets = pow2_at_least(std::max<uint64_t>(1, cdiv(P * 4, BUCKET_ENTRIES)));
    cv.ht.bucket_mask = c->n_buckets - 1;
    cv.ht.shift = 32u - (uint32_t)(bit_width(c->n_buckets) - 1);
    if ((rc = dev_alloc(c, &cv.ht.entries, (size_t)c->n_buckets * BUCKET_ENTRIES)) ||
        (rc = dev_alloc(c, &cv.ht.reach, c->n_buckets)))
        return rc;

    // workspaces
    Workspace &ws = c->ws;
    const size_t N = (size_t)max_batch_ids;
    const size_t ptiles = cdiv(N, PT_TILE);
    const size_t sort_tiles = cdiv(N, SORT_TILE);
    const size_t ap_tiles = cdiv(N, (per_lane <= 1 ? ap_tile_for(g.lanes) : 128));
    for (int set = 0; set < SORT_SETS; ++set) {
        for (int i = 0; i < 2; ++i)
            if ((rc = dev_alloc(c, &c->keys[set][i], N)) || (rc = dev_alloc(c, &c->idx[set][i], N))) return rc;
        if ((rc = dev_alloc(c, &c->sort_hist[set], sort_tiles * (SORT_MAX_BINS / 2)))) return rc;
    }
    c->cv.last = &cv.ds->call[0];
    c->cv.next_call = &cv.ds->call[1];
    if ((rc = dev_alloc(c, &ws.src, N)) || (rc = dev_alloc(c, &ws.head_slot, N)) || (rc = dev_alloc(c, &ws.cls, N)) ||
        (rc = dev_alloc(c, &ws.tile_miss, ptiles)) || (rc = dev_alloc(c, &ws.tile_stale, ptiles)) ||
        (rc = dev_alloc(c, &ws.miss_stage, ptiles * PT_TILE)) || (rc = dev_alloc(c, &ws.stale_stage, ptiles * PT_TILE)) ||
        (rc = dev_alloc(c, &c->inv, N)) || (rc = dev_alloc(c, &ws.bag_of, N)) ||
        (rc = dev_alloc(c, &c->bd.part, ap_tiles * 4 * (size_t)c->dim)) || (rc = dev_alloc(c, &c->bd.slot, ap_tiles)) ||      // (tiles' sums, then groups' sums: see ApplyBorders)
        (rc = dev_alloc(c, &c->bd.arrived, ap_tiles * 3)) || (rc = dev_alloc(c, &c->bd.from_key, ap_tiles)))
        return rc;
    const size_t slot_tiles = cdiv(P, TRIM_TILE), ev_blocks = cdiv(P, EV_SLOTS), ev_supers = cdiv(ev_blocks, EV_SUPER);
    c->tp.zero_words = (uint32_t)(SEL_MAX_PASSES * SEL_BINS + 4 * ev_supers);
    if ((rc = dev_alloc(c, &c->tp.hist, (size_t)c->tp.zero_words)) || (rc = dev_alloc(c, &c->tp.blk_cnt, ev_blocks)) ||
        (rc = dev_alloc(c, &c->tile_free[0], slot_tiles)) ||
        (rc = dev_alloc(c, &c->tile_free[1], slot_tiles)) || (rc = dev_alloc(c, &c->ev_ids[0], P)) || (rc = dev_alloc(c, &c->ev_ids[1], P)))
        return rc;
    {   // before the first trim every slot is free
        std::vector<uint32_t> full(slot_tiles);
        for (size_t t = 0; t < slot_tiles; ++t) full[t] = (uint32_t)std::min<uint64_t>(TRIM_TILE, P - t * TRIM_TILE);
        HIP_TRY(hipMemcpy(c->tile_free[0], full.data(), slot_tiles * sizeof(uint32_t), hipMemcpyHostToDevice));
    }
    HIP_TRY(hipMemsetAsync(c->tile_free[1], 0, slot_tiles * sizeof(uint32_t), c->stream));

    HIP_TRY(hipMemsetAsync(c->bd.arrived, 0, ap_tiles * 3 * sizeof(uint32_t), c->stream));
    HIP_TRY(hipMemsetAsync(cv.ds, 0, sizeof(DState), c->stream));
    init_cache_kernel<<<1024, 256, 0, c->stream>>>(cv, c->n_buckets * BUCKET_ENTRIES, c->n_buckets);
    if ((rc = launch_ok())) return rc;
    HIP_TRY(hipStreamSynchronize(c->stream));
    c->configured = true;
    return HET_OK;
}

int het_cache_configure(het_cache *c, int64_t max_batch_ids, int32_t optimizer, float eps, void *hip_stream)
{
    const size_t keep = c ? c->owned.size() : 0, mark = c ? c->arena_used : 0;
    const int rc = configure_impl(c, max_batch_ids, optimizer, eps, hip_stream);
    if (rc != HET_OK && c && !c->configured) free_owned_from(c, keep, mark);     // a retry starts from nothing
    return rc;
}

static int attach_impl(het_cache *c, float *table, float *state, uint32_t *cg, int64_t vocab, int32_t location)
{
    if (!c || !c->configured || !table || !cg || vocab <= 0 || vocab >= 0xFFFFFFFFll) return HET_EINVAL;
    if (location != HET_BACKING_HBM && location != HET_BACKING_PINNED_HOST) return HET_EINVAL;
    if (c->optimizer != HET_OPT_SGD && !state) return HET_EINVAL;
    if (c->optimizer == HET_OPT_ADAGRAD_ROWWISE && location != HET_BACKING_HBM) return HET_EINVAL;
    if (c->attached) return HET_EINVAL;
    if (c->many && location != HET_BACKING_HBM) return HET_EINVAL;      // several workers: the shared table lives in HBM
    if (location == HET_BACKING_PINNED_HOST) {
        // kernels need the device-side alias of the mapped host memory
        void *dt = nullptr, *dst = nullptr, *dcg = nullptr;
        HIP_TRY(hipHostGetDevicePointer(&dt, table, 0));
        HIP_TRY(hipHostGetDevicePointer(&dcg, cg, 0));
        if (state) HIP_TRY(hipHostGetDevicePointer(&dst, state, 0));
        table = static_cast<float *>(dt); cg = static_cast<uint32_t *>(dcg); state = static_cast<float *>(dst);
    }
    c->cv.W = table; c->cv.A = state; c->cv.Cg = cg; c->cv.Cg_host = nullptr; c->cv.vocab = (uint32_t)vocab;
    if (c->cv.direct) {
        if (vocab >= (1ll << 31)) return HET_EINVAL;        // a key stands for its own slot
        c->cv.rows = table; c->cv.acc = state;
    } else if (location == HET_BACKING_PINNED_HOST) {
        // The kernels work on a mirror of the global clocks in HBM (a probe must not cross the host
        // link for four bytes per key); the caller's array is written through.  Evicted rows are
        // staged in HBM and written back behind the step (HostLink).
        int rc;
        uint32_t *mirror = nullptr;
        if ((rc = dev_alloc(c, &mirror, (size_t)vocab))) return rc;
        HIP_TRY(hipMemcpy(mirror, cg, (size_t)vocab * sizeof(uint32_t), hipMemcpyDefault));
        c->cv.Cg_host = cg;
        c->cv.Cg = mirror;
        c->cv.early_cc = nullptr;            // (no early push over the host link: the update does not fetch there)
        HostLink &hl = c->cv.hl;
        const size_t N = (size_t)c->max_ids, row_elems = N * (size_t)c->dim;
        if ((rc = dev_alloc(c, &hl.pend, (size_t)vocab))) return rc;
        HIP_TRY(hipMemset(hl.pend, 0, (size_t)vocab * sizeof(uint64_t)));
        for (int b = 0; b < 2; ++b) {
            if ((rc = dev_alloc(c, &hl.rows[b], row_elems)) || (rc = dev_alloc(c, &hl.keys[b], N)) || (rc = dev_alloc(c, &hl.cg[b], N))) return rc;
            if (state && (rc = dev_alloc(c, &hl.acc[b], row_elems))) return rc;
        }
        if ((rc = dev_alloc(c, &hl.pf_rows, row_elems)) || (rc = dev_alloc(c, &hl.pf_keys, N)) || (rc = dev_alloc(c, &hl.pf_from, N))) return rc;
        if (state && (rc = dev_alloc(c, &hl.pf_acc, row_elems))) return rc;
        // the stream beside the main one (default priority), and the two events that order them
        HIP_TRY(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
        HIP_TRY(hipEventCreateWithFlags(&c->ev_main, hipEventDisableTiming));
        HIP_TRY(hipEventCreateWithFlags(&c->ev_link, hipEventDisableTiming));
    }
    c->location = location;
    c->attached = true;
    return HET_OK;
}

int het_attach_backing(het_cache *c, float *table, float *state, uint32_t *cg, int64_t vocab, int32_t location)
{
    const size_t keep = c ? c->owned.size() : 0, mark = c ? c->arena_used : 0;
    const bool was = c && c->attached;
    const int rc = attach_impl(c, table, state, cg, vocab, location);
    if (rc != HET_OK && c && !was) {
        free_owned_from(c, keep, mark);
        if (c->ev_main) { (void)hipEventDestroy(c->ev_main); c->ev_main = nullptr; }
        if (c->ev_link) { (void)hipEventDestroy(c->ev_link); c->ev_link = nullptr; }
        if (c->side) { (void)hipStreamDestroy(c->side); c->side = nullptr; }
    }
    return rc;
}

int het_cache_set_lfu_cap(het_cache *c, uint32_t cap)
{
    if (!c || c->configured || c->policy != HET_POLICY_LFU_LIGHT || cap == 0) return HET_EINVAL;
    c->lfu_cap = cap;
    return HET_OK;
}

int het_cache_set_many_writers(het_cache *c)
{
    if (!c || c->configured || c->policy == HET_POLICY_NONE) return HET_EINVAL;
    c->many = true;
    return HET_OK;
}

int het_backing_foreign_update(het_cache *c, const int64_t *ids, const float *deltas, int64_t n)
{
    if (!ready(c) || n < 0 || n >= (1ll << 31) || c->location != HET_BACKING_HBM) return HET_EINVAL;
    if (n == 0) return HET_OK;
    if (!ids || !deltas) return HET_EINVAL;
    const uint32_t grid = row_grid(c->cv.geom, (uint64_t)n);
    if (c->cv.geom.vec == 4) LAUNCH(c, K_MISC, foreign_update_kernel<4><<<grid, 256, 0, c->stream>>>(c->cv, ids, deltas, (uint32_t)n));
    else LAUNCH(c, K_MISC, foreign_update_kernel<1><<<grid, 256, 0, c->stream>>>(c->cv, ids, deltas, (uint32_t)n));
    return launch_ok();
}

int het_prefetch_cancel(het_cache *c)
{
    if (!c || !c->configured) return HET_EINVAL;
    // stages already enqueued read their buffer in stream order before anything enqueued from now on;
    // stages not enqueued yet never will be
    c->n_ann = 0;
    c->pf.ready = false;             // rows fetched ahead for a withdrawn batch are not used
    return HET_OK;
}

int het_prefetch(het_cache *c, const int64_t *ids, int64_t n)
{
    if (!ready(c) || n < 0 || n > c->max_ids) return HET_EINVAL;
    if (n == 0) return HET_OK;
    if (!ids) return HET_EINVAL;
    // Nothing is launched here: the kernels of the calls that follow carry the sort, stage by
    // stage, into a buffer set that neither the current order nor an earlier announcement uses.
    // With every spare set taken, the oldest announcement makes room.
    if (c->n_ann && c->ann[c->n_ann - 1].ids == ids && c->ann[c->n_ann - 1].n == (uint32_t)n) return HET_OK;   // said already
    if (c->n_ann == SORT_SETS - 1) drop_oldest_announcement(c);
    for (int set = 0; set < SORT_SETS; ++set) {
        bool taken = set == c->sort_set;
        for (int a = 0; a < c->n_ann; ++a) taken = taken || c->ann[a].set == set;
        if (taken) continue;
        Announced an;
        an.ids = ids; an.n = (uint32_t)n; an.set = set; an.next_stage = 0;
        c->ann[c->n_ann++] = an;
        break;
    }
    return HET_OK;
}

int het_lookup(het_cache *c, const int64_t *ids, int64_t n, float *out)
{
    if (!ready(c) || n < 0 || n > c->max_ids) return HET_EINVAL;
    if (n == 0) return HET_OK;
    if (!ids || !out) return HET_EINVAL;
    return c->cv.geom.vec == 4 ? run_lookup<4>(c, ids, (uint32_t)n, nullptr, 0, out)
                               : run_lookup<1>(c, ids, (uint32_t)n, nullptr, 0, out);
}

int het_lookup_pooled(het_cache *c, const int64_t *ids, int64_t n, const int64_t *offsets, int64_t n_bags, float *out)
{
    if (!ready(c) || n < 0 || n > c->max_ids) return HET_EINVAL;
    if (n == 0) return HET_OK;
    if (!ids || !out || !offsets || n_bags <= 0 || n_bags >= (1ll << 31)) return HET_EINVAL;
    return c->cv.geom.vec == 4 ? run_lookup<4>(c, ids, (uint32_t)n, offsets, (uint32_t)n_bags, out)
                               : run_lookup<1>(c, ids, (uint32_t)n, offsets, (uint32_t)n_bags, out);
}

int het_update(het_cache *c, const int64_t *ids, const float *grads, int64_t n, float lr)
{
    if (!ready(c) || n < 0 || n > c->max_ids) return HET_EINVAL;
    if (n == 0) return HET_OK;
    if (!ids || !grads) return HET_EINVAL;
    return c->cv.geom.vec == 4 ? run_update<4>(c, ids, (uint32_t)n, nullptr, 0, grads, lr)
                               : run_update<1>(c, ids, (uint32_t)n, nullptr, 0, grads, lr);
}

int het_update_pooled(het_cache *c, const int64_t *ids, int64_t n, const int64_t *offsets, const float *bag_grads,
                      int64_t n_bags, float lr)
{
    if (!ready(c) || n < 0 || n > c->max_ids) return HET_EINVAL;
    if (n == 0) return HET_OK;
    if (!ids || !bag_grads || !offsets || n_bags <= 0 || n_bags >= (1ll << 31)) return HET_EINVAL;
    return c->cv.geom.vec == 4 ? run_update<4>(c, ids, (uint32_t)n, offsets, (uint32_t)n_bags, bag_grads, lr)
                               : run_update<1>(c, ids, (uint32_t)n, offsets, (uint32_t)n_bags, bag_grads, lr);
}

int het_flush(het_cache *c)
{
    if (!ready(c)) return HET_EINVAL;
    begin_call(c);
    c->n_ann = 0;                // announcements do not outlive a flush
    c->pf.ready = false;
    wait_link(c);                // (nothing the flush writes may be overtaken by an older staged copy)
    drain_pushes(c);             // (a staged copy of a row reaches the table before anything the flush writes)
    { int rc0 = settle_fetch(c); if (rc0) return rc0; }
    const uint32_t grid = row_grid(c->cv.geom, c->cv.n_slots);
    if (c->cv.geom.vec == 4) LAUNCH(c, K_FLUSH, flush_kernel<4><<<grid, 256, 0, c->stream>>>(c->cv));
    else LAUNCH(c, K_FLUSH, flush_kernel<1><<<grid, 256, 0, c->stream>>>(c->cv));
    int rc = launch_ok();
    if (rc) return rc;
    return sync_and_status(c, nullptr);
}

int het_stats(het_cache *c, het_stats_t *out)
{
    if (!c || !c->configured || !out) return HET_EINVAL;
    DState h;
    int rc = sync_and_status(c, &h);
    if (rc == HET_EHIP) return rc;
    to_public(h.call[c->cslot], &out->last);
    to_public(h.total, &out->total);
    // between a lookup and its update the overflow is still cached; after a trim the count is the capacity at most
    out->resident = c->overflow_pending ? h.size : std::min<int64_t>(h.size, c->capacity);
    out->iteration = h.t;
    out->error_bits = (int32_t)h.err;
    return HET_OK;
}

int het_clear_error(het_cache *c)
{
    if (!c || !c->configured) return HET_EINVAL;
    { int rc0 = sync_all(c); if (rc0) return rc0; }
    HIP_TRY(hipMemset(&c->cv.ds->err, 0, sizeof(uint32_t)));
    return HET_OK;
}

int het_export_state(het_cache *c, int64_t *keys, int32_t *slots, uint32_t *cs, uint32_t *cc, uint32_t *last_use,
                     uint32_t *freq, int64_t *n_resident)
{
    if (!c || !c->configured) return HET_EINVAL;
    { int rc0 = sync_all(c); if (rc0) return rc0; }
    const size_t P = c->cv.n_slots;
    std::vector<uint32_t> k(P);
    std::vector<SlotMeta> m(P);
    HIP_TRY(hipMemcpy(k.data(), c->cv.slot_key, P * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(m.data(), c->cv.meta, P * sizeof(SlotMeta), hipMemcpyDeviceToHost));
    int64_t r = 0;
    for (size_t slot = 0; slot < P; ++slot) {
        if (k[slot] == KEY_NONE) continue;
        if (keys) keys[r] = k[slot];
        if (slots) slots[r] = (int32_t)slot;
        if (cs) cs[r] = m[slot].cs;
        if (cc) cc[r] = m[slot].cc;
        if (last_use) last_use[r] = m[slot].last_use;
        if (freq) freq[r] = m[slot].freq;
        ++r;
    }
    if (n_resident) *n_resident = r;
    return HET_OK;
}

int het_export_rows(het_cache *c, float *rows, float *acc)
{
    if (!c || !c->configured) return HET_EINVAL;
    { int rc0 = settle_fetch(c); if (rc0) return rc0; }
    { int rc0 = sync_all(c); if (rc0) return rc0; }
    const size_t P = c->cv.n_slots, D = (size_t)c->dim;
    if (c->cv.direct) return HET_OK;                 // no cache: nothing is ever cached
    std::vector<uint32_t> k(P);
    HIP_TRY(hipMemcpy(k.data(), c->cv.slot_key, P * 4, hipMemcpyDeviceToHost));
    // the slot arrays come over in a few large copies (a copy per row would be one synchronous
    // transfer per cached row) and are compacted here
    const size_t step = std::max<size_t>(1, ((size_t)64 << 20) / (D * 4));
    std::vector<float> buf(std::min(step, P) * D);
    for (int which = 0; which < 2; ++which) {
        float *dst = which ? acc : rows;
        const float *src = which ? c->cv.acc : c->cv.rows;
        if (!dst || !src) continue;
        const size_t W = which && c->cv.rowwise ? 1 : D;        // (row-wise Adagrad: one accumulator per row)
        size_t r = 0;
        for (size_t s0 = 0; s0 < P; s0 += step) {
            const size_t cnt = std::min(step, P - s0);
            bool any = false;
            for (size_t i = 0; i < cnt && !any; ++i) any = k[s0 + i] != KEY_NONE;
            if (!any) continue;
            HIP_TRY(hipMemcpy(buf.data(), src + s0 * W, cnt * W * 4, hipMemcpyDeviceToHost));
            for (size_t i = 0; i < cnt; ++i)
                if (k[s0 + i] != KEY_NONE) { std::memcpy(dst + r * W, buf.data() + i * W, W * 4); ++r; }
        }
    }
    return HET_OK;
}

int het_last_lookup(het_cache *c, int64_t *keys, int32_t *cls, int32_t *slots, int64_t *n_unique)
{
    if (!c || !c->configured) return HET_EINVAL;
    { int rc0 = sync_all(c); if (rc0) return rc0; }
    const size_t n = c->last_lookup_n;
    std::vector<uint32_t> k(n);
    std::vector<int32_t> sl(n);
    std::vector<uint8_t> cl(n);
    if (n) {
        HIP_TRY(hipMemcpy(k.data(), c->ws.skey, n * 4, hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(sl.data(), c->ws.head_slot, n * 4, hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(cl.data(), c->ws.cls, n, hipMemcpyDeviceToHost));
    }
    int64_t u = 0;
    for (size_t j = 0; j < n; ++j) {             // per-key facts sit at the head of each run
        if (k[j] == c->cv.vocab || (j > 0 && k[j] == k[j - 1])) continue;
        if (keys) keys[u] = k[j];
        if (cls) cls[u] = cl[j];
        if (slots) slots[u] = sl[j];
        ++u;
    }
    if (n_unique) *n_unique = u;
    return HET_OK;
}

int het_last_evicted(het_cache *c, int64_t *ids, int64_t *n)
{
    if (!c || !c->configured) return HET_EINVAL;
    { int rc0 = sync_all(c); if (rc0) return rc0; }
    DState h;
    HIP_TRY(hipMemcpy(&h, c->cv.ds, sizeof(DState), hipMemcpyDeviceToHost));
    const int last = c->tf_last;                         // the list the last trim filled
    const uint32_t ev_n = c->last_trim_skipped ? 0u : h.ev_n[last];
    std::vector<uint32_t> e(ev_n);
    if (ev_n) HIP_TRY(hipMemcpy(e.data(), c->ev_ids[last], (size_t)ev_n * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < e.size(); ++i)
        if (ids) ids[i] = e[i];
    if (n) *n = (int64_t)ev_n;
    return HET_OK;
}

// ---- a Read without a cache object and without any allocation ------------------------------
// Scratch of het_lookup_nocache_static: the sort's double buffers and per-tile histograms, the
// per-position workspaces of the gather and the block of device-side scalars.  One copy per GPU,
// held until the process ends; every call on a GPU uses it, so calls that overlap on one GPU race.
constexpr size_t NOALLOC_MAX_IDS = HET_NOALLOC_MAX_IDS;
constexpr size_t na_align(size_t v) { return (v + 255) & ~(size_t)255; }
constexpr size_t NA_WORDS = na_align(NOALLOC_MAX_IDS * 4);                 // one uint32 / int32 per id
constexpr size_t NA_HIST = na_align((NOALLOC_MAX_IDS / SORT_TILE) * (SORT_MAX_BINS / 2) * 4);
constexpr size_t NA_OFF_KEYS0 = 0, NA_OFF_KEYS1 = NA_OFF_KEYS0 + NA_WORDS, NA_OFF_IDX0 = NA_OFF_KEYS1 + NA_WORDS,
                 NA_OFF_IDX1 = NA_OFF_IDX0 + NA_WORDS, NA_OFF_HIST = NA_OFF_IDX1 + NA_WORDS, NA_OFF_SRC = NA_OFF_HIST + NA_HIST,
                 NA_OFF_HEAD = NA_OFF_SRC + NA_WORDS, NA_OFF_CLS = NA_OFF_HEAD + NA_WORDS,
                 NA_OFF_DS = NA_OFF_CLS + na_align(NOALLOC_MAX_IDS), NA_BYTES = NA_OFF_DS + na_align(sizeof(DState));
static __device__ __align__(256) unsigned char scratch[NA_BYTES];

__global__ void na_clear_kernel(DState *ds)
{
    uint32_t *w = reinterpret_cast<uint32_t *>(ds);
    for (uint32_t i = threadIdx.x; i < sizeof(DState) / 4; i += blockDim.x) w[i] = 0;
}
__global__ void na_report_kernel(const DState *ds, uint32_t *err_out) { *err_out = ds->err; }

constexpr int NA_MAX_DEVICES = 64;
static unsigned char *na_scratch_of_device[NA_MAX_DEVICES];      // the array's address on each GPU, asked for once

int het_lookup_nocache_static(const float *table, int64_t vocab, int32_t dim, const int64_t *ids, int64_t n, float *out,
                              uint32_t *err_bits, void *hip_stream)
{
    if (n < 0 || n > (int64_t)NOALLOC_MAX_IDS || dim <= 0 || vocab <= 0 || vocab >= (1ll << 31)) return HET_EINVAL;
    if (n == 0) return HET_OK;
    if (!table || !ids || !out) return HET_EINVAL;
    RowGeom g;
    g.dim = dim; g.vec = (dim % 4 == 0) ? 4 : 1; g.chunks = dim / g.vec;
    g.lanes = (int)std::min<uint32_t>(64u, pow2_at_least((uint64_t)g.chunks));
    if ((g.chunks + g.lanes - 1) / g.lanes > 16) return HET_EINVAL;          // rows wider than the kernels take
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= NA_MAX_DEVICES) return HET_EINVAL;
    if (!na_scratch_of_device[dev]) {
        // the array's name is a host-side handle; its device address differs from GPU to GPU
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return HET_EHIP;
        na_scratch_of_device[dev] = static_cast<unsigned char *>(p);
    }
    unsigned char *base = na_scratch_of_device[dev];
    // a cache object that lives for this call only, in the "no cache" mode, over the scratch
    het_cache tmp;
    tmp.capacity = 1; tmp.dim = dim; tmp.policy = HET_POLICY_NONE;
    tmp.configured = tmp.attached = true;
    tmp.max_ids = (int64_t)NOALLOC_MAX_IDS;
    tmp.stream = static_cast<hipStream_t>(hip_stream);
    CacheView &cv = tmp.cv;
    cv.direct = 1; cv.n_slots = 1; cv.capacity = 1; cv.max_ids = (uint32_t)NOALLOC_MAX_IDS;
    cv.geom = g;
    cv.W = const_cast<float *>(table); cv.rows = cv.W; cv.vocab = (uint32_t)vocab;
    cv.ds = reinterpret_cast<DState *>(base + NA_OFF_DS);
    cv.last = &cv.ds->call[0]; cv.next_call = &cv.ds->call[1];
    tmp.keys[0][0] = reinterpret_cast<uint32_t *>(base + NA_OFF_KEYS0);
    tmp.keys[0][1] = reinterpret_cast<uint32_t *>(base + NA_OFF_KEYS1);
    tmp.idx[0][0] = reinterpret_cast<uint32_t *>(base + NA_OFF_IDX0);
    tmp.idx[0][1] = reinterpret_cast<uint32_t *>(base + NA_OFF_IDX1);
    tmp.sort_hist[0] = reinterpret_cast<uint32_t *>(base + NA_OFF_HIST);
    tmp.ws.src = reinterpret_cast<int32_t *>(base + NA_OFF_SRC);
    tmp.ws.head_slot = reinterpret_cast<int32_t *>(base + NA_OFF_HEAD);
    tmp.ws.cls = reinterpret_cast<uint8_t *>(base + NA_OFF_CLS);
    // the scratch keeps the last call's contents: the scalars (sticky error bits, counters) start at zero
    na_clear_kernel<<<1, 64, 0, tmp.stream>>>(cv.ds);
    const int rc = g.vec == 4 ? run_lookup<4>(&tmp, ids, (uint32_t)n, nullptr, 0, out)
                              : run_lookup<1>(&tmp, ids, (uint32_t)n, nullptr, 0, out);
    if (rc != HET_OK) return rc;
    if (err_bits) na_report_kernel<<<1, 1, 0, tmp.stream>>>(cv.ds, err_bits);
    return launch_ok();
}

int het_profile_begin(het_cache *c)
{
    if (!c || !c->configured || c->profiling) return HET_EINVAL;
    c->profiling = true;
    return HET_OK;
}

int het_profile_end(het_cache *c, double *total_ms, int64_t *launches, int32_t n_kernels)
{
    if (!c || !c->profiling) return HET_EINVAL;
    c->profiling = false;
    int rc = HET_OK;
    if (sync_all(c) != HET_OK) rc = HET_EHIP;
    for (int i = 0; i < n_kernels; ++i) {
        if (total_ms) total_ms[i] = 0.0;
        if (launches) launches[i] = 0;
    }
    for (ProfSpan &sp : c->spans) {
        float ms = 0.f;
        if (rc == HET_OK && hipEventElapsedTime(&ms, sp.start, sp.stop) == hipSuccess && sp.id < n_kernels) {
            if (total_ms) total_ms[sp.id] += ms;
            if (launches) launches[sp.id] += 1;
        }
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    c->spans.clear();
    return rc;
}

int het_profile_rows(int32_t pattern, float *x, float *a, const float *src, const uint32_t *idx, int64_t n, int32_t dim,
                     const uint32_t *gidx, int32_t per, int32_t reps, double *avg_ms, void *hip_stream)
{
    if (pattern < 0 || pattern > 2 || n <= 0 || n > (int64_t)1 << 30 || dim <= 0 || dim % 4 || reps <= 0 || !avg_ms || !x) return HET_EINVAL;
    if (pattern != HET_PATTERN_UPDATE && !src) return HET_EINVAL;
    if (pattern != HET_PATTERN_COPY && !idx) return HET_EINVAL;
    if (pattern == HET_PATTERN_UPDATE && (per < 0 || per > 3 || per == 1 || (per > 0 && (!src || !gidx)))) return HET_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    const int lanes = std::min(dim / 4, 64);
    if (lanes & (lanes - 1)) return HET_EINVAL;          // (row groups of 1, 2, 4, ... 64 lanes: rows of 4, 8, 16, ... 128 floats, or wider)
    const uint32_t per_block = 256u / (uint32_t)lanes;
    const uint32_t rows_at_once = pattern == HET_PATTERN_UPDATE ? PAT_UPDATE_ROWS : PAT_ROWS;
    const uint32_t grid = std::max(1u, std::min(cdiv(cdiv((uint64_t)n, rows_at_once), per_block), 256u * 8u));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return HET_EHIP; }
    int rc = HET_OK;
    for (int rep = -2; rep < reps && rc == HET_OK; ++rep) {          // (two launches first that are not timed)
        if (rep == 0 && hipEventRecord(e0, st) != hipSuccess) rc = HET_EHIP;
        if (pattern == HET_PATTERN_UPDATE && per == 0) pattern_update_kernel<0><<<grid, 256, 0, st>>>(x, a, idx, (uint32_t)n, dim, nullptr, nullptr);
        else if (pattern == HET_PATTERN_UPDATE && per == 2) pattern_update_kernel<2><<<grid, 256, 0, st>>>(x, a, idx, (uint32_t)n, dim, src, gidx);
        else if (pattern == HET_PATTERN_UPDATE) pattern_update_kernel<3><<<grid, 256, 0, st>>>(x, a, idx, (uint32_t)n, dim, src, gidx);
        else pattern_gather_kernel<<<grid, 256, 0, st>>>(src, x, pattern == HET_PATTERN_GATHER ? idx : nullptr, (uint32_t)n, dim);
        if (hipGetLastError() != hipSuccess) rc = HET_EHIP;
    }
    float ms = 0.f;
    if (rc == HET_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                         hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) rc = HET_EHIP;
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    *avg_ms = (double)ms / reps;
    return rc;
}

int het_profile_trace(het_cache *c, int32_t kernel, uint64_t *records, int64_t capacity)
{
    if (!c || !c->configured || capacity < 0 || capacity > (int64_t)1 << 24 || (capacity > 0 && !records)) return HET_EINVAL;
    if (kernel != K_APPLY && kernel != K_FILL_GATHER) return HET_EINVAL;
    KernelTrace &t = c->trace[kernel == K_APPLY ? 0 : 1];
    t.rec = capacity ? reinterpret_cast<unsigned long long *>(records) : nullptr;
    t.cap = (uint32_t)capacity;
    return HET_OK;
}

int het_profile_kernel_count(void) { return K_NUM; }

const char *het_profile_kernel_name(int index) { return index >= 0 && index < K_NUM ? kKernelNames[index] : ""; }

int het_cache_destroy(het_cache *c)
{
    if (!c) return HET_OK;
    int rc = HET_OK;
    if (c->configured && sync_all(c) != HET_OK) rc = HET_EHIP;
    if (c->ev_main) (void)hipEventDestroy(c->ev_main);
    if (c->ev_link) (void)hipEventDestroy(c->ev_link);
    if (c->side) (void)hipStreamDestroy(c->side);
    for (void *p : c->owned)
        if (hipFree(p) != hipSuccess) rc = HET_EHIP;
    delete c;
    return rc;
}

#ifndef HET_BUILD_ID
#define HET_BUILD_ID "unknown"
#endif
const char *het_build_id(void) { return HET_BUILD_ID; }

const char *het_strerror(int status)
{
    switch (status) {
    case HET_OK: return "ok";
    case HET_EINVAL: return "invalid argument or call order";
    case HET_ENOMEM: return "out of memory";
    case HET_EHIP: return "HIP runtime error";
    case HET_ERANGE: return "an id was outside [0, vocab)";
    case HET_ESTATE: return "update of an id that is not cached";
    default: return "unknown status";
    }
}

} // extern "C"
