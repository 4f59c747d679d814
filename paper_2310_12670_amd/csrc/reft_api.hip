// C-ABI host logic of libreft (see include/reft.h): the plan (host integer arithmetic and device
// tables), the bucket pipelines that pair the gather / scatter kernels with chunked
// hipMemcpyAsync transfers, and the XOR encode / decode entry points.
#include "../../include/reft.h"
#include "reft_internal.hpp"

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <algorithm>
#include <exception>
#include <map>
#include <mutex>
#include <new>
#include <vector>

using namespace reft;

// ------------------------------------------------------------------------------------------------
// errors and tunables
// ------------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// Entry points that build host-side tables must not let an allocation failure escape the C ABI.
#define REFT_GUARD_BEGIN try {
#define REFT_GUARD_END(who)                                                                       \
    }                                                                                             \
    catch (const std::exception &e)                                                               \
    {                                                                                             \
        return fail(REFT_EINVAL, "%s: host allocation failed (%s)", who, e.what());               \
    }

#define HIPCHK(expr)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return fail(REFT_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),         \
                        __FILE__, __LINE__);                                                      \
    } while (0)

static std::atomic<uint64_t> g_max_wgs{0};       // 0 = 16 per compute unit
static std::atomic<uint64_t> g_nontemporal{1};
static std::atomic<uint64_t> g_unroll{4};
static std::atomic<uint64_t> g_tile_shift{18};   // read at plan creation
static std::atomic<uint64_t> g_host_only{0};     // read at plan creation: no device tables
static std::atomic<uint64_t> g_link_wgs{32};     // grid cap of kernels bound by the host link
static std::atomic<uint64_t> g_small_pieces{8}; // spans starting in a tile that switch it to LDS mode
static std::atomic<uint64_t> g_dma_min{65536};   // pieces of at least this many bytes are copied by DMA
static std::atomic<uint64_t> g_gather_min{8};    // shortest run of smaller pieces worth a gather kernel
static std::atomic<uint64_t> g_dma_streams{1};   // 2 = piece copies alternate with a helper stream
static std::atomic<uint64_t> g_graph_copies{0};  // piece copies as a hipGraph: 0 off, 1 independent nodes, 2 chain
static std::atomic<uint64_t> g_burst{1};         // parity encode may use the write-burst kernel
static std::atomic<uint64_t> g_burst_min_rows{5};    // ... from this many sources on
static std::atomic<uint64_t> g_burst_min_bytes{8ull << 20};  // ... and from this stream length on
static std::atomic<uint64_t> g_burst_stage{32768};   // stream bytes per workgroup and round
static std::atomic<uint64_t> g_burst_wgs{2};         // resident workgroups per compute unit
static std::atomic<uint64_t> g_burst_polls{6};       // bound on a writer wave's wait per round (0 = no waiting)
static std::atomic<uint64_t> g_burst_nap{16};        // pause between polls, units of 1024 cycles

extern "C" int reft_set_tunable(const char *name, uint64_t value)
{
    if (!name) return fail(REFT_EINVAL, "reft_set_tunable: null name");
    if (!strcmp(name, "max_wgs")) {
        if (value > (1u << 20)) return fail(REFT_EINVAL, "max_wgs out of range");
        g_max_wgs = value;
    } else if (!strcmp(name, "nontemporal")) {
        if (value > 1) return fail(REFT_EINVAL, "nontemporal must be 0 or 1");
        g_nontemporal = value;
    } else if (!strcmp(name, "unroll")) {
        if (value != 1 && value != 2 && value != 4)
            return fail(REFT_EINVAL, "unroll must be 1, 2 or 4");
        g_unroll = value;
    } else if (!strcmp(name, "tile_shift")) {
        if (value < 12 || value > 24) return fail(REFT_EINVAL, "tile_shift must be in [12, 24]");
        g_tile_shift = value;
    } else if (!strcmp(name, "link_wgs")) {
        if (value < 1 || value > (1u << 20)) return fail(REFT_EINVAL, "link_wgs out of range");
        g_link_wgs = value;
    } else if (!strcmp(name, "dma_min_bytes")) {
        g_dma_min = value;
    } else if (!strcmp(name, "dma_streams")) {
        if (value < 1 || value > 2) return fail(REFT_EINVAL, "dma_streams must be 1 or 2");
        g_dma_streams = value;
    } else if (!strcmp(name, "graph_copies")) {
        if (value > 2) return fail(REFT_EINVAL, "graph_copies must be 0, 1 or 2");
        g_graph_copies = value;
    } else if (!strcmp(name, "gather_min_pieces")) {
        if (value < 1) return fail(REFT_EINVAL, "gather_min_pieces must be at least 1");
        g_gather_min = value;
    } else if (!strcmp(name, "small_pieces")) {
        if (value > 0xffffffffull) return fail(REFT_EINVAL, "small_pieces out of range");
        g_small_pieces = value;
    } else if (!strcmp(name, "host_only_plans")) {
        if (value > 1) return fail(REFT_EINVAL, "host_only_plans must be 0 or 1");
        g_host_only = value;
    } else if (!strcmp(name, "burst")) {
        if (value > 1) return fail(REFT_EINVAL, "burst must be 0 or 1");
        g_burst = value;
    } else if (!strcmp(name, "burst_min_rows")) {
        if (value < 1) return fail(REFT_EINVAL, "burst_min_rows must be at least 1");
        g_burst_min_rows = value;
    } else if (!strcmp(name, "burst_min_bytes")) {
        g_burst_min_bytes = value;
    } else if (!strcmp(name, "burst_stage_bytes")) {
        if (value < 4096 || value > 65536 || value % 4096)
            return fail(REFT_EINVAL, "burst_stage_bytes must be a multiple of 4096 in [4096, 65536]");
        g_burst_stage = value;
    } else if (!strcmp(name, "burst_wgs_per_cu")) {
        if (value < 1 || value > 8) return fail(REFT_EINVAL, "burst_wgs_per_cu must be in [1, 8]");
        g_burst_wgs = value;
    } else if (!strcmp(name, "burst_max_polls")) {
        if (value > 100000) return fail(REFT_EINVAL, "burst_max_polls must be at most 100000");
        g_burst_polls = value;
    } else if (!strcmp(name, "burst_nap")) {
        if (value > 1024) return fail(REFT_EINVAL, "burst_nap must be at most 1024");
        g_burst_nap = value;

    } else {
        return fail(REFT_EINVAL, "unknown tunable '%s'", name);
    }
    return REFT_OK;
}

extern "C" int reft_get_tunable(const char *name, uint64_t *value)
{
    if (!name || !value) return fail(REFT_EINVAL, "reft_get_tunable: null argument");
    if (!strcmp(name, "max_wgs")) *value = g_max_wgs;
    else if (!strcmp(name, "nontemporal")) *value = g_nontemporal;
    else if (!strcmp(name, "unroll")) *value = g_unroll;
    else if (!strcmp(name, "tile_shift")) *value = g_tile_shift;
    else if (!strcmp(name, "host_only_plans")) *value = g_host_only;
    else if (!strcmp(name, "link_wgs")) *value = g_link_wgs;
    else if (!strcmp(name, "small_pieces")) *value = g_small_pieces;
    else if (!strcmp(name, "dma_min_bytes")) *value = g_dma_min;
    else if (!strcmp(name, "gather_min_pieces")) *value = g_gather_min;
    else if (!strcmp(name, "dma_streams")) *value = g_dma_streams;
    else if (!strcmp(name, "graph_copies")) *value = g_graph_copies;
    else if (!strcmp(name, "burst")) *value = g_burst;
    else if (!strcmp(name, "burst_min_rows")) *value = g_burst_min_rows;
    else if (!strcmp(name, "burst_min_bytes")) *value = g_burst_min_bytes;
    else if (!strcmp(name, "burst_stage_bytes")) *value = g_burst_stage;
    else if (!strcmp(name, "burst_wgs_per_cu")) *value = g_burst_wgs;
    else if (!strcmp(name, "burst_max_polls")) *value = g_burst_polls;
    else if (!strcmp(name, "burst_nap")) *value = g_burst_nap;
    else return fail(REFT_EINVAL, "unknown tunable '%s'", name);
    return REFT_OK;
}

extern "C" const char *reft_last_error(void) { return g_err; }
extern "C" const char *reft_version(void) { return "libreft 0.1 (gfx950)"; }

// ------------------------------------------------------------------------------------------------
// plan
// ------------------------------------------------------------------------------------------------
namespace {
constexpr int kRing = 32;       // pointer tables the plan's cache holds at once
constexpr int kUsers = 4;       // streams per cached table whose most recent use is tracked
constexpr uint32_t kRingRows = 72;  // capacity of the cache, in rows of T pointers (>= 2 * (REFT_MAX_K + 1))
constexpr int kMaxSlots = 64;   // staging slots used by the staged bucket pipelines
constexpr int kGroups = 2;      // the slots form two groups that alternate (double buffering)
constexpr uint32_t kCtrBlocks = 8;  // burst launches that may be in flight on one ring of counters
constexpr size_t kPieceLists = 8;   // classified bucket ranges a plan remembers

struct Event {
    hipEvent_t ev = nullptr;
    bool recorded = false;
};

struct Run {            // stream range [a, b) of consecutive small pieces: gather kernel + one copy
    uint64_t a, b;
};
struct Dma {            // one piece (bucket x span) copied by the DMA path straight from its tensor
    uint64_t o, n, span;
};
// How the bytes of a bucket range travel in the staged transport (see classify_pieces); depends
// on the plan and two tunables only, so it is computed once and kept.
struct PieceLists {
    uint64_t b0 = 0, b1 = 0, dma_min = 0, gather_min = 0, tick = 0;
    std::vector<Run> runs;
    std::vector<Dma> dmas;
};

// One cached pointer table: `len` pointers at position `pos` of the plan's pool (pinned host
// mirror and device copy).  `uploaded` is recorded behind the host-to-device copy; used[i] behind
// the last kernel that read the table on stream user[i].
struct PtrEntry {
    bool live = false;
    uint64_t pos = 0, len = 0, hash = 0, tick = 0;
    hipStream_t up_stream = nullptr;
    Event uploaded;
    hipStream_t user[kUsers] = {};
    Event used[kUsers];
};

// A plan derived from a base plan for the rotated placement, with the recipe that turns the
// caller's pointers into its rows: entry (w * T' + t) says where piece t of window w starts.
struct RowRecipe {
    uint32_t span;      // span of the base plan, or kContig / kZeros
    uint64_t add;       // byte offset inside that span (or inside the contiguous operand)
};
constexpr uint32_t kContig = 0xffffffffu, kZeros = 0xfffffffeu;
}  // namespace

struct DerivedPlan {
    reft_plan *plan = nullptr;
    uint32_t nwin = 0;
    std::vector<RowRecipe> recipe;
};

struct reft_plan {
    bool host_only = false;           // sizing only: no device tables, data calls are refused
    int device = 0;
    int num_cus = 256;
    uint64_t T = 0, NB = 0, L = 0, max_bucket = 0;
    uint32_t tile_shift = 16;
    uint64_t ntiles = 0;
    std::vector<uint64_t> off;        // [T+1]
    std::vector<uint64_t> bstart;     // [NB+1]
    std::vector<uint32_t> first;      // [ntiles] host copy of the tile table
    uint64_t *d_off = nullptr;
    uint32_t *d_first = nullptr;
    // cache of pointer tables: a pool of ring_cap pointers (pinned host mirror and device copy)
    // handed out front to back, and the tables that currently live in it
    uint64_t ring_cap = 0, ring_head = 0, ring_tick = 0;
    uint64_t *h_ptr = nullptr;
    uint64_t *d_ptr = nullptr;
    PtrEntry ring[kRing];
    // host scratch for the row tables of the XOR entry points ((REFT_MAX_K + 1) * T pointers)
    std::vector<const void *> row_buf;
    // classified piece lists of recent bucket ranges (the whole stream's is made at creation)
    std::vector<PieceLists> pieces;
    uint64_t pieces_tick = 0;
    // stream on which the most recent snapshot's completion event was recorded
    hipStream_t last_pack_stream = nullptr;
    // device address of the library's static scratch on this plan's GPU (see reft_parity_encode_noalloc)
    unsigned char *scratch = nullptr;
    // bucket pipelines
    Event pack_filled[kGroups], pack_free[kGroups], pack_done, pack_begin, rest_begin;
    Event rest_filled[kGroups], rest_free[kGroups], rest_done, rest_copied;
    // helper stream for the staged transport's piece copies (tunable "dma_streams" = 2), default
    // priority, and the events that fork it from / join it to copy_stream
    hipStream_t aux = nullptr;
    Event aux_fork, aux_join;
    // rotated parity placement: plans derived from this one (merged piece lists of shifted
    // windows), keyed by (kind, k, member, segment), and a small all-zero device buffer that
    // stands in for the zero extension of the last segment
    std::map<uint64_t, DerivedPlan> derived;
    void *zeros = nullptr;
    // the piece copies of recent snapshot / restore calls as instantiated graphs (see copy_graph)
    struct CopyGraph {
        std::vector<uint64_t> key;
        hipGraphExec_t exec = nullptr;
        uint64_t used = 0;
        hipEvent_t done = nullptr;    // recorded behind the most recent launch
    };
    std::vector<CopyGraph> graphs;
    uint64_t graph_tick = 0;
    // write-burst kernel: spans that start in each tile, sorted (plans with many tiles dense in
    // small spans keep the ordinary kernel), and a ring of counter blocks, one per launch in flight
    std::vector<uint32_t> tile_spans_sorted;
    uint32_t *burst_ctr = nullptr;
    uint32_t burst_next = 0;

    PlanTables tables() const { return PlanTables{d_off, d_first, T, L, tile_shift}; }
};

static LaunchCfg launch_cfg(const reft_plan *p)
{
    uint64_t w = g_max_wgs;
    if (w == 0) w = 16ull * (uint64_t)(p ? p->num_cus : 256);
    return LaunchCfg{(uint32_t)w, (uint32_t)g_unroll.load(), g_nontemporal.load() != 0,
                     (uint32_t)g_small_pieces.load()};
}

// Kernels whose rate is set by the host link need only a few workgroups to saturate it.
static LaunchCfg link_cfg(const reft_plan *p)
{
    LaunchCfg c = launch_cfg(p);
    const uint64_t w = g_link_wgs.load();
    if (w < c.max_wgs) c.max_wgs = (uint32_t)w;
    return c;
}

// The address at which the GPU sees a host buffer, or 0 if it is not mapped for device access
// (pageable memory).  Clears the sticky error a failed lookup leaves behind.
static uint64_t device_view_of_host(const void *host)
{
    void *d = nullptr;
    if (hipHostGetDevicePointer(&d, const_cast<void *>(host), 0) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return (uint64_t)(uintptr_t)d;
}

static int make_event(Event &e)
{
    HIPCHK(hipEventCreateWithFlags(&e.ev, hipEventDisableTiming));
    e.recorded = false;
    return REFT_OK;
}

static int record(Event &e, hipStream_t s)
{
    HIPCHK(hipEventRecord(e.ev, s));
    e.recorded = true;
    return REFT_OK;
}

static int wait_on(hipStream_t s, const Event &e)
{
    if (e.recorded) HIPCHK(hipStreamWaitEvent(s, e.ev, 0));
    return REFT_OK;
}

// ------------------------------------------------------------------------------------------------
// static device memory of the library
// ------------------------------------------------------------------------------------------------
// `scratch` serves reft_parity_encode_noalloc, the entry point for callers that cannot allocate:
// a table of up to kScratchPtrs span pointers, then one block of burst counters.  Every GPU the
// library runs on holds its own copy until the process ends.  `static_ctr` is the ring of counter
// blocks of reft_reconstruct, which has no plan to keep them in.  In host code these names are
// stand-ins, not device addresses: the addresses come from hipGetSymbolAddress, once per device.
constexpr uint32_t kScratchPtrs = 32768;
constexpr size_t kScratchPtrBytes = (size_t)kScratchPtrs * sizeof(uint64_t);
constexpr size_t kScratchBytes = kScratchPtrBytes + 2560;            // 256 KiB + counters
static_assert(kBurstCtrBytes <= 2560, "the counter block must fit behind the pointer table");
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static __device__ __align__(256) uint32_t static_ctr[kCtrBlocks * (kBurstCtrBytes / sizeof(uint32_t))];

namespace {
constexpr int kMaxDevices = 64;
struct DeviceStatics {
    bool known = false;
    unsigned char *scratch = nullptr;
    uint32_t *ctr = nullptr;
    int num_cus = 256;
};
std::mutex g_statics_mu;
DeviceStatics g_statics[kMaxDevices];
}  // namespace

// The addresses of the static arrays on the current device (resolved on first use per device).
static int device_statics(const DeviceStatics **out)
{
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(REFT_EINVAL, "GPU %d: unsupported device index", dev);
    std::lock_guard<std::mutex> lock(g_statics_mu);
    DeviceStatics &d = g_statics[dev];
    if (!d.known) {
        void *a = nullptr, *b = nullptr;
        HIPCHK(hipGetSymbolAddress(&a, HIP_SYMBOL(scratch)));
        HIPCHK(hipGetSymbolAddress(&b, HIP_SYMBOL(static_ctr)));
        if (!a || !b) return fail(REFT_EHIP, "hipGetSymbolAddress returned a null address");
        hipDeviceProp_t prop;
        HIPCHK(hipGetDeviceProperties(&prop, dev));
        d.scratch = (unsigned char *)a;
        d.ctr = (uint32_t *)b;
        d.num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        d.known = true;
    }
    *out = &d;
    return REFT_OK;
}

// ------------------------------------------------------------------------------------------------
// cache of pointer tables
// ------------------------------------------------------------------------------------------------
static void free_ring(reft_plan *p)
{
    if (p->h_ptr) (void)hipHostFree(p->h_ptr);
    if (p->d_ptr) (void)hipFree(p->d_ptr);
    p->h_ptr = nullptr;
    p->d_ptr = nullptr;
    p->ring_cap = 0;
}

static uint64_t hash_ptrs(const void *const *ptrs, size_t n)
{
    uint64_t h = 0x9e3779b97f4a7c15ull ^ n;
    for (size_t i = 0; i < n; ++i) {
        h ^= (uint64_t)(uintptr_t)ptrs[i];
        h *= 0x100000001b3ull;
        h ^= h >> 29;
    }
    return h;
}

// The host waits for exactly the work that may still read the entry's table (its upload and the
// kernels behind which a use was recorded): never for the whole device.
static int retire_entry(PtrEntry &e)
{
    if (e.uploaded.recorded) HIPCHK(hipEventSynchronize(e.uploaded.ev));
    e.uploaded.recorded = false;
    for (int i = 0; i < kUsers; ++i) {
        if (e.used[i].recorded) HIPCHK(hipEventSynchronize(e.used[i].ev));
        e.used[i].recorded = false;
        e.user[i] = nullptr;
    }
    e.live = false;
    return REFT_OK;
}

// Make `rows` x T pointers available on the device: reuse the cached table that already holds
// exactly these pointers (a trainer passes the same tensors every iteration; a stream other than
// the one that uploaded it waits for the upload only), else take the next room in the pool,
// retiring the tables that lie there, and start the upload on `s`.  On success *dev_tab is the
// device table and *entry the cache index to pass to release_ptrs after the last kernel that
// reads the table.
static int upload_ptrs(reft_plan *p, const void *const *ptrs, uint32_t rows, hipStream_t s,
                       const uint64_t **dev_tab, int *entry)
{
    static_assert(sizeof(void *) == sizeof(uint64_t), "pointers are 64-bit");
    const uint64_t n = (uint64_t)rows * p->T;
    if (n > p->ring_cap)
        return fail(REFT_ESIZE, "pointer table of %u rows exceeds the plan's cache (%llu pointers)",
                    rows, (unsigned long long)p->ring_cap);
    const uint64_t h = hash_ptrs(ptrs, n);
    int rc;
    for (int i = 0; i < kRing; ++i) {
        PtrEntry &e = p->ring[i];
        if (e.live && e.len == n && e.hash == h &&
            !memcmp(p->h_ptr + e.pos, ptrs, n * sizeof(uint64_t))) {
            if (e.up_stream != s && e.uploaded.recorded)
                HIPCHK(hipStreamWaitEvent(s, e.uploaded.ev, 0));
            e.tick = ++p->ring_tick;
            *dev_tab = p->d_ptr + e.pos;
            *entry = i;
            return REFT_OK;
        }
    }
    const uint64_t pos = p->ring_head + n > p->ring_cap ? 0 : p->ring_head;
    int slot = -1;
    for (int i = 0; i < kRing; ++i) {
        PtrEntry &e = p->ring[i];
        if (e.live && e.pos < pos + n && pos < e.pos + e.len && (rc = retire_entry(e))) return rc;
        if (!e.live && slot < 0) slot = i;
    }
    if (slot < 0) {                                    // every slot is live: the oldest goes
        slot = 0;
        for (int i = 1; i < kRing; ++i)
            if (p->ring[i].tick < p->ring[slot].tick) slot = i;
        if ((rc = retire_entry(p->ring[slot]))) return rc;
    }
    PtrEntry &e = p->ring[slot];
    memcpy(p->h_ptr + pos, ptrs, n * sizeof(uint64_t));
    HIPCHK(hipMemcpyAsync(p->d_ptr + pos, p->h_ptr + pos, n * sizeof(uint64_t),
                          hipMemcpyHostToDevice, s));
    HIPCHK(hipEventRecord(e.uploaded.ev, s));
    e.uploaded.recorded = true;
    e.up_stream = s;
    e.live = true;
    e.pos = pos;
    e.len = n;
    e.hash = h;
    e.tick = ++p->ring_tick;
    p->ring_head = pos + n;
    *dev_tab = p->d_ptr + pos;
    *entry = slot;
    return REFT_OK;
}

// Record, on stream s, that the kernels queued so far were the last ones to read entry's table.
static int release_ptrs(reft_plan *p, int entry, hipStream_t s)
{
    PtrEntry &e = p->ring[entry];
    int i = -1;
    for (int u = 0; u < kUsers && i < 0; ++u)
        if (e.used[u].recorded && e.user[u] == s) i = u;
    for (int u = 0; u < kUsers && i < 0; ++u)
        if (!e.used[u].recorded) i = u;
    for (int u = 0; u < kUsers && i < 0; ++u)
        if (hipEventQuery(e.used[u].ev) == hipSuccess) i = u;
    if (i < 0) {                                       // more streams than tracked: wait for one
        i = 0;
        HIPCHK(hipEventSynchronize(e.used[0].ev));
    }
    (void)hipGetLastError();                           // hipEventQuery's "not ready" is no error
    e.user[i] = s;
    HIPCHK(hipEventRecord(e.used[i].ev, s));
    e.used[i].recorded = true;
    return REFT_OK;
}

static int check_plan(const reft_plan *p, const char *who)
{
    if (!p) return fail(REFT_EINVAL, "%s: null plan", who);
    if (p->host_only)
        return fail(REFT_EINVAL, "%s: the plan was created host-only (no device tables)", who);
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev != p->device)
        return fail(REFT_EINVAL, "%s: plan belongs to GPU %d but GPU %d is current", who,
                    p->device, dev);
    return REFT_OK;
}

static int check_span_ptrs(const reft_plan *p, const void *const *ptrs, uint32_t rows,
                           const char *who)
{
    if (!ptrs) return fail(REFT_EINVAL, "%s: null pointer array", who);
    for (uint32_t r = 0; r < rows; ++r)
        for (uint64_t t = 0; t < p->T; ++t)
            if (!ptrs[r * p->T + t] && p->off[t + 1] != p->off[t])
                return fail(REFT_EINVAL, "%s: span %llu of shard %u is null but has %llu bytes",
                            who, (unsigned long long)t, r,
                            (unsigned long long)(p->off[t + 1] - p->off[t]));
    return REFT_OK;
}

static const PieceLists &pieces_of(reft_plan *p, uint64_t b0, uint64_t b1);

extern "C" int reft_plan_create(const uint64_t *span_nbytes, uint64_t T,
                                const uint64_t *bucket_nbytes, uint64_t NB,
                                uint64_t uniform_bucket, reft_plan **out)
{
    REFT_GUARD_BEGIN
    if (!out) return fail(REFT_EINVAL, "reft_plan_create: null out");
    *out = nullptr;
    if (!span_nbytes || T == 0) return fail(REFT_EINVAL, "reft_plan_create: no spans");
    if (T >= 0xffffffffull) return fail(REFT_EINVAL, "reft_plan_create: too many spans");

    reft_plan *p = new (std::nothrow) reft_plan;
    if (!p) return fail(REFT_EINVAL, "reft_plan_create: out of host memory");
    struct Guard {
        reft_plan *p;
        ~Guard() { if (p) reft_plan_destroy(p); }
    } guard{p};

    p->T = T;
    p->off.resize(T + 1);
    p->off[0] = 0;
    for (uint64_t t = 0; t < T; ++t)
        if (__builtin_add_overflow(p->off[t], span_nbytes[t], &p->off[t + 1]))
            return fail(REFT_ESIZE, "reft_plan_create: stream length overflows 64 bits");
    p->L = p->off[T];

    // buckets
    p->bstart.push_back(0);
    if (uniform_bucket) {
        for (uint64_t b = 0; b < p->L; b += uniform_bucket)
            p->bstart.push_back(b + uniform_bucket < p->L ? b + uniform_bucket : p->L);
    } else if (!bucket_nbytes && NB == 0) {
        if (p->L) p->bstart.push_back(p->L);              // no bucketing asked: one bucket
    } else {
        if (NB && !bucket_nbytes) return fail(REFT_EINVAL, "reft_plan_create: null bucket list");
        uint64_t acc = 0;
        for (uint64_t b = 0; b < NB; ++b) {
            if (bucket_nbytes[b] == 0)
                return fail(REFT_EINVAL, "reft_plan_create: bucket %llu has zero length",
                            (unsigned long long)b);
            if (__builtin_add_overflow(acc, bucket_nbytes[b], &acc) || acc > p->L)
                return fail(REFT_ESIZE, "reft_plan_create: buckets exceed the stream length");
            p->bstart.push_back(acc);
        }
        if (acc != p->L)
            return fail(REFT_ESIZE, "reft_plan_create: buckets cover %llu of %llu stream bytes",
                        (unsigned long long)acc, (unsigned long long)p->L);
    }
    p->NB = p->bstart.size() - 1;
    for (uint64_t b = 0; b < p->NB; ++b)
        if (p->bstart[b + 1] - p->bstart[b] > p->max_bucket)
            p->max_bucket = p->bstart[b + 1] - p->bstart[b];

    // tile table: first span that owns a byte of tile t (zero-length spans never qualify)
    p->tile_shift = (uint32_t)g_tile_shift.load();
    const uint64_t tile = 1ull << p->tile_shift;
    p->ntiles = (p->L + tile - 1) >> p->tile_shift;
    std::vector<uint32_t> &first = p->first;
    first.assign(p->ntiles ? p->ntiles : 1, 0);
    {
        uint64_t i = 0;
        for (uint64_t t = 0; t < p->ntiles; ++t) {
            const uint64_t o = t << p->tile_shift;
            while (p->off[i + 1] <= o) ++i;      // o < L = off[T] keeps i < T
            first[t] = (uint32_t)i;
        }
        p->tile_spans_sorted.resize(p->ntiles);
        for (uint64_t t = 0; t < p->ntiles; ++t) {
            const uint64_t nxt = t + 1 < p->ntiles ? first[t + 1] : T - 1;
            p->tile_spans_sorted[t] = (uint32_t)(nxt - first[t]);
        }
        std::sort(p->tile_spans_sorted.begin(), p->tile_spans_sorted.end());
    }

    if (g_host_only.load()) {
        p->host_only = true;
        guard.p = nullptr;
        *out = p;
        return REFT_OK;
    }
    HIPCHK(hipGetDevice(&p->device));
    hipDeviceProp_t prop;
    HIPCHK(hipGetDeviceProperties(&prop, p->device));
    p->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    HIPCHK(hipMalloc((void **)&p->d_off, (T + 1) * sizeof(uint64_t)));
    HIPCHK(hipMalloc((void **)&p->d_first, first.size() * sizeof(uint32_t)));
    HIPCHK(hipMemcpy(p->d_off, p->off.data(), (T + 1) * sizeof(uint64_t), hipMemcpyHostToDevice));
    HIPCHK(hipMemcpy(p->d_first, first.data(), first.size() * sizeof(uint32_t),
                     hipMemcpyHostToDevice));
    HIPCHK(hipMalloc((void **)&p->burst_ctr, kCtrBlocks * kBurstCtrBytes));
    int rc;
    const DeviceStatics *ds = nullptr;
    if ((rc = device_statics(&ds))) return rc;
    p->scratch = ds->scratch;
    for (int i = 0; i < kRing; ++i) {
        if ((rc = make_event(p->ring[i].uploaded))) return rc;
        for (int u = 0; u < kUsers; ++u)
            if ((rc = make_event(p->ring[i].used[u]))) return rc;
    }
    for (int i = 0; i < kGroups; ++i) {
        if ((rc = make_event(p->pack_filled[i])) || (rc = make_event(p->pack_free[i])) ||
            (rc = make_event(p->rest_filled[i])) || (rc = make_event(p->rest_free[i])))
            return rc;
    }
    if ((rc = make_event(p->pack_done)) || (rc = make_event(p->rest_done)) ||
        (rc = make_event(p->rest_copied)) || (rc = make_event(p->pack_begin)) ||
        (rc = make_event(p->rest_begin)) || (rc = make_event(p->aux_fork)) ||
        (rc = make_event(p->aux_join)))
        return rc;
    // The helper stream exists only where it is asked for: a stream takes its place among the
    // process's few hardware queues when it is created, whether it ever gets work or not (two
    // idle helper streams made here were enough to push a snapshot and a restore, on streams
    // created after them, onto one queue, where they took turns on the link).
    if (g_dma_streams.load() == 2) HIPCHK(hipStreamCreateWithFlags(&p->aux, hipStreamNonBlocking));
    // everything a data-moving call needs is made here: the pointer-table pool, the host scratch
    // for row tables, and the whole stream's piece lists for the staged transport
    p->ring_cap = (uint64_t)kRingRows * T;
    HIPCHK(hipHostMalloc((void **)&p->h_ptr, p->ring_cap * sizeof(uint64_t), hipHostMallocDefault));
    HIPCHK(hipMalloc((void **)&p->d_ptr, p->ring_cap * sizeof(uint64_t)));
    p->row_buf.resize((size_t)(REFT_MAX_K + 1) * T);
    p->pieces.reserve(kPieceLists);
    (void)pieces_of(p, 0, p->NB);

    guard.p = nullptr;
    *out = p;
    return REFT_OK;
    REFT_GUARD_END("reft_plan_create")
}

extern "C" void reft_plan_destroy(reft_plan *p)
{
    if (!p) return;
    // let everything that still reads the plan's tables finish
    auto drain = [](Event &e) {
        if (e.ev) {
            if (e.recorded) (void)hipEventSynchronize(e.ev);
            (void)hipEventDestroy(e.ev);
            e.ev = nullptr;
        }
    };
    for (int i = 0; i < kRing; ++i) {
        drain(p->ring[i].uploaded);
        for (int u = 0; u < kUsers; ++u) drain(p->ring[i].used[u]);
    }
    for (int i = 0; i < kGroups; ++i) {
        drain(p->pack_filled[i]);
        drain(p->pack_free[i]);
        drain(p->rest_filled[i]);
        drain(p->rest_free[i]);
    }
    drain(p->pack_done);
    drain(p->rest_done);
    drain(p->rest_copied);
    drain(p->aux_fork);
    drain(p->aux_join);
    if (p->aux) (void)hipStreamDestroy(p->aux);
    drain(p->pack_begin);
    drain(p->rest_begin);
    free_ring(p);
    for (auto &g : p->graphs) {
        if (g.done) {
            (void)hipEventSynchronize(g.done);
            (void)hipEventDestroy(g.done);
        }
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
    }
    if (p->burst_ctr) (void)hipFree(p->burst_ctr);
    for (auto &kv : p->derived) reft_plan_destroy(kv.second.plan);
    p->derived.clear();
    if (p->zeros) (void)hipFree(p->zeros);
    if (p->d_off) (void)hipFree(p->d_off);
    if (p->d_first) (void)hipFree(p->d_first);
    delete p;
}

extern "C" uint64_t reft_plan_stream_bytes(const reft_plan *p) { return p ? p->L : 0; }
extern "C" uint64_t reft_plan_num_spans(const reft_plan *p) { return p ? p->T : 0; }
extern "C" uint64_t reft_plan_num_buckets(const reft_plan *p) { return p ? p->NB : 0; }
extern "C" uint64_t reft_plan_max_bucket_bytes(const reft_plan *p) { return p ? p->max_bucket : 0; }

static uint64_t slot_stride(const reft_plan *p)
{
    // room for the bucket plus the sub-256-byte phase that keeps slot addresses congruent to
    // stream offsets (so 16-byte-aligned spans stay aligned in the slot)
    return (p->max_bucket + 256 + 255) & ~255ull;
}

extern "C" uint64_t reft_plan_staging_slot_bytes(const reft_plan *p)
{
    return p ? slot_stride(p) : 0;
}

extern "C" int reft_plan_bucket_range(const reft_plan *p, uint64_t b, uint64_t *begin,
                                      uint64_t *end)
{
    if (!p || !begin || !end) return fail(REFT_EINVAL, "reft_plan_bucket_range: null argument");
    if (b >= p->NB) return fail(REFT_EINVAL, "reft_plan_bucket_range: bucket %llu of %llu",
                                (unsigned long long)b, (unsigned long long)p->NB);
    *begin = p->bstart[b];
    *end = p->bstart[b + 1];
    return REFT_OK;
}

extern "C" int reft_plan_tile_info(const reft_plan *p, uint64_t *tile_bytes, uint64_t *ntiles)
{
    if (!p || !tile_bytes || !ntiles) return fail(REFT_EINVAL, "reft_plan_tile_info: null argument");
    *tile_bytes = 1ull << p->tile_shift;
    *ntiles = p->ntiles;
    return REFT_OK;
}

extern "C" int reft_plan_tile_first_span(const reft_plan *p, uint64_t t, uint64_t *span)
{
    if (!p || !span) return fail(REFT_EINVAL, "reft_plan_tile_first_span: null argument");
    if (t >= p->ntiles) return fail(REFT_EINVAL, "reft_plan_tile_first_span: tile out of range");
    *span = p->first[t];
    return REFT_OK;
}

extern "C" int reft_plan_span_offset(const reft_plan *p, uint64_t t, uint64_t *offset)
{
    if (!p || !offset) return fail(REFT_EINVAL, "reft_plan_span_offset: null argument");
    if (t > p->T) return fail(REFT_EINVAL, "reft_plan_span_offset: span out of range");
    *offset = p->off[t];
    return REFT_OK;
}

extern "C" int reft_plan_split(const reft_plan *p, double t_bubble, double t_ss, uint64_t *cut)
{
    if (!p || !cut) return fail(REFT_EINVAL, "reft_plan_split: null argument");
    if (!(t_ss > 0.0) || !(t_bubble >= 0.0))
        return fail(REFT_EINVAL, "reft_plan_split: need t_ss > 0 and t_bubble >= 0");
    const long double x = (long double)p->L * ((long double)t_bubble / (long double)t_ss);
    *cut = x >= (long double)p->L ? p->L : (uint64_t)x;   // floor, clamped to L
    return REFT_OK;
}

extern "C" int reft_plan_staged_work(reft_plan *p, uint64_t *gather_launches, uint64_t *copies)
{
    REFT_GUARD_BEGIN
    if (!p || !gather_launches || !copies)
        return fail(REFT_EINVAL, "reft_plan_staged_work: null argument");
    const PieceLists &pl = pieces_of(p, 0, p->NB);
    *gather_launches = pl.runs.size();
    *copies = pl.runs.size() + pl.dmas.size();
    return REFT_OK;
    REFT_GUARD_END("reft_plan_staged_work")
}

extern "C" int reft_plan_burst_stats(reft_plan *p, uint64_t stats[4])
{
    int rc = check_plan(p, "reft_plan_burst_stats");
    if (rc) return rc;
    if (!stats) return fail(REFT_EINVAL, "reft_plan_burst_stats: null argument");
    stats[0] = stats[1] = stats[2] = stats[3] = 0;
    if (p->burst_next == 0) return REFT_OK;              // no burst launch on this plan yet
    const uint32_t slot = (p->burst_next - 1) % kCtrBlocks;
    const uint32_t *blk = p->burst_ctr + (size_t)slot * (kBurstCtrBytes / sizeof(uint32_t));
    uint32_t w[4] = {0, 0, 0, 0};
    HIPCHK(hipDeviceSynchronize());                      // a diagnostic: the launch must have ended
    HIPCHK(hipMemcpy(w, blk + kBurstDiagWord, 3 * sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIPCHK(hipMemcpy(w + 3, blk + 8 * 64, sizeof(uint32_t), hipMemcpyDeviceToHost));
    for (int i = 0; i < 4; ++i) stats[i] = w[i];
    return REFT_OK;
}

// ------------------------------------------------------------------------------------------------
// how the bytes of a bucket range travel between the tensors and the host (staged transport)
// ------------------------------------------------------------------------------------------------
// A piece of at least dma_min bytes needs no kernel: the runtime's copy engines move it between
// the tensor and the host buffer, which costs kernels running beside it next to nothing.  Smaller
// pieces are worth a copy of their own only when few of them lie together; a run of at least
// gather_min consecutive small pieces inside one bucket is gathered into a staging slot by one
// kernel launch and leaves as one copy (many small tensors would otherwise mean thousands of tiny
// transfers).
static void classify_pieces(const reft_plan *p, uint64_t bucket_begin, uint64_t bucket_end,
                            uint64_t dma_min, uint64_t gather_min, std::vector<Run> &runs,
                            std::vector<Dma> &dmas)
{
    std::vector<Dma> pending;
    auto flush = [&]() {
        if (pending.empty()) return;
        if (pending.size() >= gather_min)
            runs.push_back(Run{pending.front().o, pending.back().o + pending.back().n});
        else
            dmas.insert(dmas.end(), pending.begin(), pending.end());
        pending.clear();
    };
    uint64_t i = 0;
    for (uint64_t b = bucket_begin; b < bucket_end; ++b) {
        const uint64_t lo = p->bstart[b], hi = p->bstart[b + 1];
        if (b == bucket_begin) {
            // the span that owns byte lo: last one with off <= lo that is not empty
            uint64_t l = 0, h = p->T;
            while (h - l > 1) {
                const uint64_t m = (l + h) / 2;
                if (p->off[m] <= lo) l = m;
                else h = m;
            }
            i = l;
        }
        for (uint64_t o = lo; o < hi;) {
            while (p->off[i + 1] <= o) ++i;              // o < hi <= L = off[T]
            const uint64_t pe = p->off[i + 1] < hi ? p->off[i + 1] : hi;
            // (a piece carried over from the previous bucket, see below, leaves now unless the
            // bucket's first piece is the large rest of its span: a run never crosses a bucket)
            if (o == lo && !pending.empty() &&
                !(pe - o >= dma_min && pending.back().span == i &&
                  pending.back().o + pending.back().n == o))
                flush();
            // A bucket boundary is no reason to split a copy that needs no staging: a piece that
            // continues the previous copy's span is added to that copy, and a small first piece of
            // a span is carried into the large one that follows it.
            if (pending.empty() && !dmas.empty() && dmas.back().span == i &&
                dmas.back().o + dmas.back().n == o && dmas.back().n >= dma_min) {
                dmas.back().n += pe - o;
            } else if (pe - o >= dma_min) {
                uint64_t start = o;
                if (!pending.empty() && pending.back().span == i &&
                    pending.back().o + pending.back().n == o) {
                    start = pending.back().o;
                    pending.pop_back();
                }
                flush();
                dmas.push_back(Dma{start, pe - start, i});
            } else {
                pending.push_back(Dma{o, pe - o, i});
            }
            o = pe;
        }
        // a run never crosses a bucket; a single small piece at the bucket's end may still be
        // the head of a span that continues in the next bucket
        if (pending.size() == 1 && b + 1 < bucket_end && p->off[pending.back().span + 1] > hi)
            continue;
        flush();
    }
    flush();
}

// The piece lists of buckets [b0, b1) under the current tunables: made once per range and kept
// (the least recently used of kPieceLists ranges goes when another one is asked for).
static const PieceLists &pieces_of(reft_plan *p, uint64_t b0, uint64_t b1)
{
    const uint64_t dma_min = g_dma_min.load(), gather_min = g_gather_min.load();
    for (auto &pl : p->pieces)
        if (pl.b0 == b0 && pl.b1 == b1 && pl.dma_min == dma_min && pl.gather_min == gather_min) {
            pl.tick = ++p->pieces_tick;
            return pl;
        }
    PieceLists *pl = nullptr;
    p->pieces.reserve(kPieceLists);                     // references handed out stay valid
    if (p->pieces.size() < kPieceLists) {
        p->pieces.emplace_back();
        pl = &p->pieces.back();
    } else {
        pl = &p->pieces[0];
        for (auto &q : p->pieces)
            if (q.tick < pl->tick) pl = &q;
        pl->runs.clear();
        pl->dmas.clear();
    }
    pl->b0 = b0;
    pl->b1 = b1;
    pl->dma_min = dma_min;
    pl->gather_min = gather_min;
    pl->tick = ++p->pieces_tick;
    classify_pieces(p, b0, b1, dma_min, gather_min, pl->runs, pl->dmas);
    return *pl;
}

// The piece copies of a call as one hipGraph of memcpy nodes, launched on copy_stream.  A trainer
// snapshots the same tensors into the same host buffer every time, so the graph is built once
// (keyed by direction, host buffer, bucket range and the span pointers) and replayed: the
// runtime then issues the copies without a host call each, and independent nodes may use more
// than one copy engine (2106 copies of 8 KiB ... 11 MiB, 11.8 GB: 52.6 GB/s as stream copies,
// 54.7 as a chain of nodes, 55.6 as independent nodes; one copy of everything: 57.0).  Off by
// default: two such graphs launched on two streams do not run side by side, so a snapshot and a
// restore that should share the link in both directions take turns instead.
constexpr size_t kCopyGraphs = 8;

static int copy_graph(reft_plan *p, const std::vector<Dma> &dmas, hipStream_t cs, bool to_host,
                      const void *host_base, const void *const *span_ptrs, uint64_t mode)
{
    std::vector<uint64_t> key;
    key.reserve(4 + 3 * dmas.size());
    key.push_back(to_host ? 1 : 0);
    key.push_back((uint64_t)(uintptr_t)host_base);
    key.push_back(mode);
    key.push_back(dmas.size());
    for (const Dma &d : dmas) {
        key.push_back(d.o);
        key.push_back(d.n);
        key.push_back((uint64_t)(uintptr_t)span_ptrs[d.span]);
    }
    reft_plan::CopyGraph *hit = nullptr;
    for (auto &g : p->graphs)
        if (g.key == key) hit = &g;
    if (!hit) {
        hipGraph_t graph = nullptr;
        HIPCHK(hipGraphCreate(&graph, 0));
        struct Guard {
            hipGraph_t g;
            ~Guard() { (void)hipGraphDestroy(g); }
        } guard{graph};
        hipGraphNode_t prev = nullptr;
        for (const Dma &d : dmas) {
            uint8_t *dev = (uint8_t *)span_ptrs[d.span] + (d.o - p->off[d.span]);
            uint8_t *host = (uint8_t *)host_base + d.o;
            hipGraphNode_t node = nullptr;
            HIPCHK(hipGraphAddMemcpyNode1D(&node, graph, mode == 2 && prev ? &prev : nullptr,
                                           mode == 2 && prev ? 1 : 0, to_host ? (void *)host : (void *)dev,
                                           to_host ? (const void *)dev : (const void *)host, d.n,
                                           to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice));
            prev = node;
        }
        hipGraphExec_t exec = nullptr;
        HIPCHK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
        if (p->graphs.size() >= kCopyGraphs) {
            // the least recently used one goes; it may still be running
            size_t lru = 0;
            for (size_t i = 1; i < p->graphs.size(); ++i)
                if (p->graphs[i].used < p->graphs[lru].used) lru = i;
            HIPCHK(hipEventSynchronize(p->graphs[lru].done));
            (void)hipGraphExecDestroy(p->graphs[lru].exec);
            (void)hipEventDestroy(p->graphs[lru].done);
            p->graphs.erase(p->graphs.begin() + (long)lru);
        }
        hipEvent_t done = nullptr;
        HIPCHK(hipEventCreateWithFlags(&done, hipEventDisableTiming));
        p->graphs.push_back(reft_plan::CopyGraph{std::move(key), exec, 0, done});
        hit = &p->graphs.back();
    }
    hit->used = ++p->graph_tick;
    HIPCHK(hipGraphLaunch(hit->exec, cs));
    HIPCHK(hipEventRecord(hit->done, cs));
    return REFT_OK;
}

// Issue the piece copies on copy_stream, or alternately on copy_stream and the plan's helper
// stream (forked from and joined back to copy_stream, so ordering on copy_stream still covers
// every copy): two queues hide the set-up gap between consecutive small copies.
template <typename Issue>
static int issue_piece_copies(reft_plan *p, const std::vector<Dma> &dmas, hipStream_t cs, Issue issue)
{
    int rc;
    const bool two = g_dma_streams.load() == 2 && dmas.size() >= 4;
    if (two) {
        // made with the plan when "dma_streams" was 2 then, else on the first call that wants it
        if (!p->aux) HIPCHK(hipStreamCreateWithFlags(&p->aux, hipStreamNonBlocking));
        if ((rc = record(p->aux_fork, cs))) return rc;
        if ((rc = wait_on(p->aux, p->aux_fork))) return rc;
    }
    for (size_t i = 0; i < dmas.size(); ++i) HIPCHK(issue(dmas[i], (two && (i & 1)) ? p->aux : cs));
    if (two) {
        if ((rc = record(p->aux_join, p->aux))) return rc;
        if ((rc = wait_on(cs, p->aux_join))) return rc;
    }
    return REFT_OK;
}

// ------------------------------------------------------------------------------------------------
// S1 + S2 + S3: snapshot
// ------------------------------------------------------------------------------------------------
// Record the snapshot completion event behind the call's last work.  The event covers every
// snapshot call issued on the plan so far: when the previous call ended on another stream, this
// one's completion also waits (on the device) for that call's.
static int record_pack_done(reft_plan *p, hipStream_t s)
{
    int rc;
    if (p->pack_done.recorded && p->last_pack_stream != s && (rc = wait_on(s, p->pack_done))) return rc;
    p->last_pack_stream = s;
    return record(p->pack_done, s);
}

static int staging_slots(const reft_plan *p, const void *staging, uint64_t staging_bytes,
                         const char *who, int *nslots)
{
    if (p->NB == 0) {
        *nslots = 1;
        return REFT_OK;
    }
    if (!staging) return fail(REFT_EINVAL, "%s: null staging buffer", who);
    if ((uintptr_t)staging & 255)
        return fail(REFT_EINVAL, "%s: staging buffer must be 256-byte aligned", who);
    const uint64_t n = staging_bytes / slot_stride(p);
    if (n < 1)
        return fail(REFT_ESIZE, "%s: staging has %llu bytes, one slot needs %llu", who,
                    (unsigned long long)staging_bytes, (unsigned long long)slot_stride(p));
    *nslots = n > (uint64_t)kMaxSlots ? kMaxSlots : (int)n;
    return REFT_OK;
}

extern "C" int reft_snapshot_pack_range(reft_plan *p, const void *const *span_ptrs, void *staging,
                                        uint64_t staging_bytes, void *host_dst, uint64_t host_cap,
                                        uint64_t bucket_begin, uint64_t bucket_end,
                                        reft_stream pack_stream, reft_stream copy_stream)
{
    REFT_GUARD_BEGIN
    int rc = check_plan(p, "reft_snapshot_pack");
    if (rc) return rc;
    if (bucket_begin > bucket_end || bucket_end > p->NB)
        return fail(REFT_EINVAL, "reft_snapshot_pack: bucket range [%llu, %llu) outside [0, %llu]",
                    (unsigned long long)bucket_begin, (unsigned long long)bucket_end,
                    (unsigned long long)p->NB);
    if ((rc = check_span_ptrs(p, span_ptrs, 1, "reft_snapshot_pack"))) return rc;
    if (host_cap < p->L)
        return fail(REFT_ESIZE, "reft_snapshot_pack: host buffer holds %llu bytes, stream has %llu",
                    (unsigned long long)host_cap, (unsigned long long)p->L);
    if (p->L && !host_dst) return fail(REFT_EINVAL, "reft_snapshot_pack: null host buffer");
    hipStream_t ps = (hipStream_t)pack_stream, cs = (hipStream_t)copy_stream;
    const PlanTables pt = p->tables();
    const uint64_t *tab = nullptr;
    int entry = 0;

    if (!staging) {
        // Direct path: the gather kernel stores straight into the pinned host buffer over the
        // host link, one launch per bucket, in order on pack_stream.  No staging, no DMA.
        const uint64_t hview = p->L ? device_view_of_host(host_dst) : 0;
        if (p->L && !hview)
            return fail(REFT_EINVAL, "reft_snapshot_pack: host buffer is not mapped for device "
                                     "access (not pinned); pass a staging ring to copy it by DMA");
        if ((rc = upload_ptrs(p, span_ptrs, 1, ps, &tab, &entry))) return rc;
        const LaunchCfg cfg = link_cfg(p);
        for (uint64_t b = bucket_begin; b < bucket_end; ++b)
            HIPCHK(launch_gather(pt, tab, 1, false, nullptr, hview, p->bstart[b], p->bstart[b + 1],
                                 cfg, ps));
        if ((rc = release_ptrs(p, entry, ps))) return rc;
        return record_pack_done(p, ps);
    }

    // Staged transport.  Large pieces go by DMA straight from their tensors; runs of small pieces
    // are gathered into staging slots and leave as one copy each (see classify_pieces).  The slots
    // form two groups that alternate between the streams; the streams meet only once per group
    // (cross-stream events are costly when thousands are in flight).
    int nslots = 1;
    if ((rc = staging_slots(p, staging, staging_bytes, "reft_snapshot_pack", &nslots))) return rc;
    const PieceLists &pl = pieces_of(p, bucket_begin, bucket_end);
    const std::vector<Run> &runs = pl.runs;
    const std::vector<Dma> &dmas = pl.dmas;
    const uint64_t stride = slot_stride(p);
    // The tensors are read on both streams.  The caller orders pack_stream behind whatever
    // produced them; copy_stream joins pack_stream here so the same ordering covers its copies.
    if (ps != cs) {
        if ((rc = record(p->pack_begin, ps))) return rc;
        if ((rc = wait_on(cs, p->pack_begin))) return rc;
    }
    if (!runs.empty()) {
        if ((rc = upload_ptrs(p, span_ptrs, 1, ps, &tab, &entry))) return rc;
        const LaunchCfg cfg = launch_cfg(p);
        const int ngroups = nslots >= kGroups ? kGroups : 1;
        const uint64_t per_group = (uint64_t)(nslots / ngroups);
        uint64_t batch = 0;
        for (uint64_t r0 = 0; r0 < runs.size(); r0 += per_group, ++batch) {
            const int g = (int)(batch % (uint64_t)ngroups);
            const uint64_t r1 = r0 + per_group < runs.size() ? r0 + per_group : runs.size();
            // the group's previous occupants must have left for the host
            if ((rc = wait_on(ps, p->pack_free[g]))) return rc;
            for (uint64_t r = r0; r < r1; ++r) {
                const uint64_t slot = (uint64_t)g * per_group + (r - r0);
                const uint64_t slot_addr =
                    (uint64_t)(uintptr_t)staging + slot * stride + (runs[r].a & 255);
                HIPCHK(launch_gather(pt, tab, 1, false, nullptr, slot_addr - runs[r].a, runs[r].a,
                                     runs[r].b, cfg, ps));
            }
            if ((rc = record(p->pack_filled[g], ps))) return rc;
            if ((rc = wait_on(cs, p->pack_filled[g]))) return rc;
            for (uint64_t r = r0; r < r1; ++r) {
                const uint64_t slot = (uint64_t)g * per_group + (r - r0);
                const uint64_t slot_addr =
                    (uint64_t)(uintptr_t)staging + slot * stride + (runs[r].a & 255);
                HIPCHK(hipMemcpyAsync((uint8_t *)host_dst + runs[r].a,
                                      (const void *)(uintptr_t)slot_addr, runs[r].b - runs[r].a,
                                      hipMemcpyDeviceToHost, cs));
            }
            if ((rc = record(p->pack_free[g], cs))) return rc;
        }
        if ((rc = release_ptrs(p, entry, ps))) return rc;
    }
    const uint64_t gmode = g_graph_copies.load();
    if (gmode && g_dma_streams.load() == 1 && dmas.size() >= 8) {
        if ((rc = copy_graph(p, dmas, cs, true, host_dst, span_ptrs, gmode))) return rc;
    } else if ((rc = issue_piece_copies(p, dmas, cs, [&](const Dma &d, hipStream_t st) {
                   return hipMemcpyAsync((uint8_t *)host_dst + d.o,
                                         (const uint8_t *)span_ptrs[d.span] + (d.o - p->off[d.span]),
                                         d.n, hipMemcpyDeviceToHost, st);
               })))
        return rc;
    // completion: every copy above is on copy_stream, the gathered ones behind their kernels
    return record_pack_done(p, cs);
    REFT_GUARD_END("reft_snapshot_pack")
}

extern "C" int reft_snapshot_pack(reft_plan *p, const void *const *span_ptrs, void *staging,
                                  uint64_t staging_bytes, void *host_dst, uint64_t host_cap,
                                  reft_stream pack_stream, reft_stream copy_stream)
{
    return reft_snapshot_pack_range(p, span_ptrs, staging, staging_bytes, host_dst, host_cap, 0,
                                    p ? p->NB : 0, pack_stream, copy_stream);
}

extern "C" int reft_plan_bucket_of(const reft_plan *p, uint64_t offset, uint64_t *bucket)
{
    if (!p || !bucket) return fail(REFT_EINVAL, "reft_plan_bucket_of: null argument");
    if (offset > p->L) return fail(REFT_EINVAL, "reft_plan_bucket_of: offset beyond the stream");
    // number of buckets that end at or before `offset` = index of the bucket holding it
    uint64_t lo = 0, hi = p->NB;
    while (lo < hi) {
        const uint64_t mid = (lo + hi) / 2;
        if (p->bstart[mid + 1] <= offset) lo = mid + 1;
        else hi = mid;
    }
    *bucket = lo;
    return REFT_OK;
}

extern "C" int reft_snapshot_wait(reft_plan *p)
{
    int rc = check_plan(p, "reft_snapshot_wait");
    if (rc) return rc;
    if (p->pack_done.recorded) HIPCHK(hipEventSynchronize(p->pack_done.ev));
    return REFT_OK;
}

extern "C" int reft_snapshot_query(reft_plan *p)
{
    int rc = check_plan(p, "reft_snapshot_query");
    if (rc) return rc;
    if (!p->pack_done.recorded) return 1;
    hipError_t e = hipEventQuery(p->pack_done.ev);
    if (e == hipSuccess) return 1;
    if (e == hipErrorNotReady) return 0;
    return fail(REFT_EHIP, "hipEventQuery failed: %s", hipGetErrorString(e));
}

// ------------------------------------------------------------------------------------------------
// completed / ongoing snapshot pair
// ------------------------------------------------------------------------------------------------
struct reft_ckpt {
    reft_plan *plan = nullptr;
    void *buf[2] = {nullptr, nullptr};
    uint64_t cap = 0;
    // pinned, device-visible: committed[i] = generation whose every byte has landed in buf[i]
    uint64_t *committed = nullptr;
    uint64_t begun[2] = {0, 0};      // generation most recently started in buf[i] (host side)
    uint64_t generation = 0;
    int ongoing = -1;                // buffer of the snapshot in progress, -1 if none
    Event committed_ev[2];           // recorded behind the commit kernel of buf[i]
};

// 1 if a commit has been queued into buffer i and has not landed yet, 0 if not, negative on error.
static int commit_pending(reft_ckpt *c, int i)
{
    if (!c->committed_ev[i].recorded) return 0;
    const hipError_t e = hipEventQuery(c->committed_ev[i].ev);
    if (e == hipSuccess) {
        c->committed_ev[i].recorded = false;
        return 0;
    }
    if (e == hipErrorNotReady) {
        (void)hipGetLastError();
        return 1;
    }
    return fail(REFT_EHIP, "hipEventQuery failed: %s", hipGetErrorString(e));
}

__global__ void k_commit(uint64_t *slot, uint64_t generation)
{
    // runs after every transfer queued before it on its stream; the store is visible to the host
    __hip_atomic_store(slot, generation, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

extern "C" int reft_ckpt_create(reft_plan *p, void *host_buf0, void *host_buf1, uint64_t cap,
                                reft_ckpt **out)
{
    if (!out) return fail(REFT_EINVAL, "reft_ckpt_create: null out");
    *out = nullptr;
    int rc = check_plan(p, "reft_ckpt_create");
    if (rc) return rc;
    if (!host_buf0 || !host_buf1 || host_buf0 == host_buf1)
        return fail(REFT_EINVAL, "reft_ckpt_create: need two distinct host buffers");
    if (cap < p->L) return fail(REFT_ESIZE, "reft_ckpt_create: buffers hold %llu bytes, stream has %llu",
                                (unsigned long long)cap, (unsigned long long)p->L);
    reft_ckpt *c = new (std::nothrow) reft_ckpt;
    if (!c) return fail(REFT_EINVAL, "reft_ckpt_create: out of host memory");
    c->plan = p;
    c->buf[0] = host_buf0;
    c->buf[1] = host_buf1;
    c->cap = cap;
    hipError_t e = hipHostMalloc((void **)&c->committed, 2 * sizeof(uint64_t), hipHostMallocDefault);
    if (e != hipSuccess) {
        delete c;
        return fail(REFT_EHIP, "hipHostMalloc failed: %s", hipGetErrorString(e));
    }
    c->committed[0] = c->committed[1] = 0;
    for (int i = 0; i < 2; ++i)
        if ((rc = make_event(c->committed_ev[i]))) {
            reft_ckpt_destroy(c);
            return rc;
        }
    *out = c;
    return REFT_OK;
}

extern "C" void reft_ckpt_destroy(reft_ckpt *c)
{
    if (!c) return;
    // a commit kernel that is still queued stores into the flags: let it finish first
    for (int i = 0; i < 2; ++i)
        if (c->committed_ev[i].ev) {
            if (c->committed_ev[i].recorded) (void)hipEventSynchronize(c->committed_ev[i].ev);
            (void)hipEventDestroy(c->committed_ev[i].ev);
        }
    if (c->committed) (void)hipHostFree(c->committed);
    delete c;
}

extern "C" int reft_ckpt_wait(reft_ckpt *c)
{
    if (!c) return fail(REFT_EINVAL, "reft_ckpt_wait: null argument");
    for (int i = 0; i < 2; ++i)
        if (c->committed_ev[i].recorded) {
            HIPCHK(hipEventSynchronize(c->committed_ev[i].ev));
            c->committed_ev[i].recorded = false;
        }
    return REFT_OK;
}

static uint64_t committed_of(const reft_ckpt *c, int i)
{
    return __atomic_load_n(&c->committed[i], __ATOMIC_ACQUIRE);
}

// Index of the newest buffer whose snapshot is complete and not being overwritten, or -1.
static int latest_complete(const reft_ckpt *c, uint64_t *gen)
{
    int best = -1;
    uint64_t best_gen = 0;
    for (int i = 0; i < 2; ++i) {
        const uint64_t g = committed_of(c, i);
        if (g != 0 && g == c->begun[i] && g > best_gen) {
            best = i;
            best_gen = g;
        }
    }
    if (gen) *gen = best_gen;
    return best;
}

extern "C" int reft_ckpt_begin(reft_ckpt *c, void **host_dst, uint64_t *generation)
{
    if (!c || !host_dst) return fail(REFT_EINVAL, "reft_ckpt_begin: null argument");
    // While a commit is in flight its buffer is neither complete nor free, and overwriting the
    // other one would leave no complete snapshot should that commit never land.
    for (int i = 0; i < 2; ++i) {
        const int pend = commit_pending(c, i);
        if (pend < 0) return pend;
        if (pend)
            return fail(REFT_EBUSY, "reft_ckpt_begin: the commit of generation %llu has not landed "
                                    "yet (reft_ckpt_wait blocks until it has)",
                        (unsigned long long)c->begun[i]);
    }
    // write into the buffer that does not hold the newest complete snapshot
    const int keep = latest_complete(c, nullptr);
    const int i = keep == 0 ? 1 : 0;
    c->generation += 1;
    c->begun[i] = c->generation;     // from here until its commit lands, buffer i counts as torn
    c->ongoing = i;
    *host_dst = c->buf[i];
    if (generation) *generation = c->generation;
    return REFT_OK;
}

extern "C" int reft_ckpt_commit(reft_ckpt *c, reft_stream stream)
{
    if (!c) return fail(REFT_EINVAL, "reft_ckpt_commit: null argument");
    if (c->ongoing < 0) return fail(REFT_EINVAL, "reft_ckpt_commit: no snapshot was begun");
    int rc = check_plan(c->plan, "reft_ckpt_commit");
    if (rc) return rc;
    hipLaunchKernelGGL(k_commit, dim3(1), dim3(1), 0, (hipStream_t)stream,
                       c->committed + c->ongoing, c->begun[c->ongoing]);
    HIPCHK(hipGetLastError());
    if ((rc = record(c->committed_ev[c->ongoing], (hipStream_t)stream))) return rc;
    c->ongoing = -1;
    return REFT_OK;
}

extern "C" int reft_ckpt_latest(reft_ckpt *c, const void **host_src, uint64_t *generation)
{
    if (!c || !host_src) return fail(REFT_EINVAL, "reft_ckpt_latest: null argument");
    uint64_t g = 0;
    const int i = latest_complete(c, &g);
    *host_src = i < 0 ? nullptr : c->buf[i];
    if (generation) *generation = g;
    return REFT_OK;
}

// ------------------------------------------------------------------------------------------------
// S1 / S7 between device buffers
// ------------------------------------------------------------------------------------------------
extern "C" int reft_pack_device(reft_plan *p, const void *const *span_ptrs, void *dst_dev,
                                uint64_t dst_cap, reft_stream stream)
{
    int rc = check_plan(p, "reft_pack_device");
    if (rc) return rc;
    if ((rc = check_span_ptrs(p, span_ptrs, 1, "reft_pack_device"))) return rc;
    if (dst_cap < p->L) return fail(REFT_ESIZE, "reft_pack_device: destination too small");
    if (p->L == 0) return REFT_OK;
    if (!dst_dev) return fail(REFT_EINVAL, "reft_pack_device: null destination");
    hipStream_t s = (hipStream_t)stream;
    const uint64_t *tab = nullptr;
    int entry = 0;
    if ((rc = upload_ptrs(p, span_ptrs, 1, s, &tab, &entry))) return rc;
    HIPCHK(launch_gather(p->tables(), tab, 1, false, nullptr, (uint64_t)(uintptr_t)dst_dev, 0, p->L,
                         launch_cfg(p), s));
    return release_ptrs(p, entry, s);
}

extern "C" int reft_unpack_device(reft_plan *p, const void *src_dev, uint64_t src_bytes,
                                  void *const *span_ptrs, reft_stream stream)
{
    int rc = check_plan(p, "reft_unpack_device");
    if (rc) return rc;
    if ((rc = check_span_ptrs(p, span_ptrs, 1, "reft_unpack_device"))) return rc;
    if (src_bytes != p->L)
        return fail(REFT_ESIZE, "reft_unpack_device: source has %llu bytes, stream has %llu",
                    (unsigned long long)src_bytes, (unsigned long long)p->L);
    if (p->L == 0) return REFT_OK;
    if (!src_dev) return fail(REFT_EINVAL, "reft_unpack_device: null source");
    hipStream_t s = (hipStream_t)stream;
    const uint64_t *tab = nullptr;
    int entry = 0;
    if ((rc = upload_ptrs(p, span_ptrs, 1, s, &tab, &entry))) return rc;
    HIPCHK(launch_scatter(p->tables(), tab, (uint64_t)(uintptr_t)src_dev, 0, p->L, launch_cfg(p),
                          s));
    return release_ptrs(p, entry, s);
}

// ------------------------------------------------------------------------------------------------
// S4: parity over span tables
// ------------------------------------------------------------------------------------------------
static BurstCfg burst_cfg(uint32_t *ring, uint32_t slot, int num_cus)
{
    BurstCfg bc;
    bc.ctr = ring + (size_t)slot * (kBurstCtrBytes / sizeof(uint32_t));
    bc.stage_bytes = (uint32_t)g_burst_stage.load();
    bc.wgs_per_cu = (uint32_t)g_burst_wgs.load();
    bc.num_cus = (uint32_t)num_cus;
    bc.max_polls = (uint32_t)g_burst_polls.load();
    bc.nap = (uint32_t)g_burst_nap.load();
    return bc;
}

// Tiles of the plan in which at least `small_pieces` spans start.
static uint64_t dense_tiles(const reft_plan *p, uint32_t small_pieces)
{
    const auto &v = p->tile_spans_sorted;
    return (uint64_t)(v.end() - std::lower_bound(v.begin(), v.end(), small_pieces));
}


// The XOR passes over a device table of `nrows` rows of span pointers (row stride T of plan p)
// into a contiguous destination or, if dtab is given, into the destination's own spans (dst_row
// is the host copy of that row, used to decide which kernel applies).  More than kMaxSrc rows
// are folded in passes.  ctr_ring holds ctr_blocks blocks of burst counters; *ctr_next picks one.
static int xor_passes(reft_plan *p, const uint64_t *tab, uint32_t nrows, const uint64_t *dtab,
                      const void *const *dst_row, void *dst_contig, uint32_t *ctr_ring,
                      uint32_t ctr_blocks, uint32_t *ctr_next, hipStream_t s)
{
    const uint64_t T = p->T;
    const LaunchCfg cfg = launch_cfg(p);
    const PlanTables pt = p->tables();
    // Passes over many rows separate reads and writes in time with the burst kernel.  It walks a
    // stage piece by piece, which is slow where many small spans lie together (the ordinary
    // kernel's LDS-staged path serves those better): plans with more than one such tile in a
    // hundred keep the ordinary kernel.  So do ragged destinations whose spans are not all
    // aligned alike relative to their stream offsets, which the staging image cannot represent.
    uint64_t vb = (uint64_t)(uintptr_t)dst_contig;
    bool burst_ok = g_burst.load() && p->L >= g_burst_min_bytes.load() &&
                    dense_tiles(p, cfg.small_pieces) * 100 <= p->ntiles;
    if (burst_ok && dst_row) {
        bool have = false;
        for (uint64_t t = 0; t < T && burst_ok; ++t) {
            if (p->off[t + 1] == p->off[t]) continue;
            const uint64_t c = ((uint64_t)(uintptr_t)dst_row[t] - p->off[t]) & 15u;
            if (!have) { vb = c; have = true; }
            else burst_ok = c == vb;
        }
    }
    uint32_t done = 0;
    while (done < nrows) {
        const bool acc = done > 0;
        uint32_t n = nrows - done;
        const uint32_t cap = (uint32_t)kMaxSrc - (acc ? 1u : 0u);
        if (n > cap) n = cap;
        if (burst_ok && n + (acc ? 1u : 0u) >= g_burst_min_rows.load()) {
            BurstCfg bc = burst_cfg(ctr_ring, (*ctr_next)++ % ctr_blocks, p->num_cus);
            HIPCHK(launch_gather_burst(pt, tab + (uint64_t)done * T, (int)n, acc, dtab, vb, 0, p->L,
                                       cfg, bc, s));
        } else {
            HIPCHK(launch_gather(pt, tab + (uint64_t)done * T, (int)n, acc, dtab,
                                 (uint64_t)(uintptr_t)dst_contig, 0, p->L, cfg, s));
        }
        done += n;
    }
    return REFT_OK;
}

// XOR of `nrows` host rows of span pointers into a contiguous destination or, if dst_row is
// given, into the destination's own spans.  The rows are uploaded as one table through the
// plan's cache (rows and dst_row may lie in the plan's row_buf).
static int xor_rows(reft_plan *p, const void *const *rows, uint32_t nrows, const void *const *dst_row,
                    void *dst_contig, hipStream_t s)
{
    int rc;
    const uint64_t T = p->T;
    const uint64_t *tab = nullptr;
    int entry = 0;
    if (dst_row) {
        // one table: the source rows, then the destination row
        const void **all = p->row_buf.data();
        if (rows != all) std::copy(rows, rows + (size_t)nrows * T, all);
        if (dst_row != all + (size_t)nrows * T) std::copy(dst_row, dst_row + T, all + (size_t)nrows * T);
        if ((rc = upload_ptrs(p, all, nrows + 1, s, &tab, &entry))) return rc;
    } else {
        if ((rc = upload_ptrs(p, rows, nrows, s, &tab, &entry))) return rc;
    }
    const uint64_t *dtab = dst_row ? tab + (uint64_t)nrows * T : nullptr;
    if ((rc = xor_passes(p, tab, nrows, dtab, dst_row, dst_contig, p->burst_ctr, kCtrBlocks,
                         &p->burst_next, s)))
        return rc;
    return release_ptrs(p, entry, s);
}

extern "C" int reft_parity_encode(reft_plan *p, const void *const *shard_span_ptrs, uint32_t k,
                                  void *parity_dev, reft_stream stream)
{
    REFT_GUARD_BEGIN
    int rc = check_plan(p, "reft_parity_encode");
    if (rc) return rc;
    if (k < 1 || k > REFT_MAX_K)
        return fail(REFT_EINVAL, "reft_parity_encode: k = %u outside [1, %d]", k, REFT_MAX_K);
    if ((rc = check_span_ptrs(p, shard_span_ptrs, k, "reft_parity_encode"))) return rc;
    if (p->L == 0) return REFT_OK;
    if (!parity_dev) return fail(REFT_EINVAL, "reft_parity_encode: null parity buffer");
    return xor_rows(p, shard_span_ptrs, k, nullptr, parity_dev, (hipStream_t)stream);
    REFT_GUARD_END("reft_parity_encode")
}

// S1 + S4 in one pass: the parity of the k shards and the packed stream of shard `own`.
extern "C" int reft_parity_encode_pack(reft_plan *p, const void *const *shard_span_ptrs, uint32_t k,
                                       uint32_t own, void *parity_dev, void *packed_dev,
                                       uint64_t packed_cap, reft_stream stream)
{
    REFT_GUARD_BEGIN
    int rc = check_plan(p, "reft_parity_encode_pack");
    if (rc) return rc;
    if (k < 1 || k > REFT_MAX_K)
        return fail(REFT_EINVAL, "reft_parity_encode_pack: k = %u outside [1, %d]", k, REFT_MAX_K);
    if (own >= k) return fail(REFT_EINVAL, "reft_parity_encode_pack: own = %u but k = %u", own, k);
    if ((rc = check_span_ptrs(p, shard_span_ptrs, k, "reft_parity_encode_pack"))) return rc;
    if (packed_cap < p->L) return fail(REFT_ESIZE, "reft_parity_encode_pack: packed buffer too small");
    if (p->L == 0) return REFT_OK;
    if (!parity_dev || !packed_dev)
        return fail(REFT_EINVAL, "reft_parity_encode_pack: null parity or packed buffer");
    hipStream_t s = (hipStream_t)stream;
    const uint64_t T = p->T;
    // the own shard's row first: the fused kernel packs the first row it reads
    const void **rows = p->row_buf.data();
    std::copy(shard_span_ptrs + (size_t)own * T, shard_span_ptrs + (size_t)(own + 1) * T, rows);
    for (uint32_t j = 0, r = 1; j < k; ++j)
        if (j != own) {
            std::copy(shard_span_ptrs + (size_t)j * T, shard_span_ptrs + (size_t)(j + 1) * T,
                      rows + (size_t)r * T);
            ++r;
        }
    const LaunchCfg cfg = launch_cfg(p);
    const uint64_t vb = (uint64_t)(uintptr_t)parity_dev, vb2 = (uint64_t)(uintptr_t)packed_dev;
    const uint64_t stage = g_burst_stage.load();
    // The fused kernel applies where the burst kernel does (rows, bytes, no tiles dense in small
    // spans), in one pass of at most kMaxSrc rows, with both destinations aligned alike and its
    // one instantiation per row count (unroll 4, non-temporal); its two LDS images per half must
    // fit a compute unit's LDS.  Otherwise: the encode and the pack as two launches.
    const bool fused = g_burst.load() && p->L >= g_burst_min_bytes.load() && k <= (uint32_t)kMaxSrc &&
                       k >= g_burst_min_rows.load() && dense_tiles(p, cfg.small_pieces) * 100 <= p->ntiles &&
                       ((vb ^ vb2) & 15u) == 0 && cfg.unroll == 4 && cfg.nontemporal &&
                       4 * (stage + 16) + 16 <= 160 * 1024;
    const uint64_t *tab = nullptr;
    int entry = 0;
    if ((rc = upload_ptrs(p, rows, k, s, &tab, &entry))) return rc;
    if (fused) {
        const BurstCfg bc = burst_cfg(p->burst_ctr, p->burst_next++ % kCtrBlocks, p->num_cus);
        HIPCHK(launch_gather_burst_pack(p->tables(), tab, (int)k, vb, vb2, 0, p->L, cfg, bc, s));
    } else {
        if ((rc = xor_passes(p, tab, k, nullptr, nullptr, parity_dev, p->burst_ctr, kCtrBlocks,
                             &p->burst_next, s)))
            return rc;
        HIPCHK(launch_gather(p->tables(), tab, 1, false, nullptr, vb2, 0, p->L, cfg, s));
    }
    return release_ptrs(p, entry, s);
    REFT_GUARD_END("reft_parity_encode_pack")
}

// ------------------------------------------------------------------------------------------------
// S4 for callers that cannot allocate
// ------------------------------------------------------------------------------------------------
namespace {
constexpr uint32_t kPtrChunk = 256;
struct PtrChunk {
    uint64_t p[kPtrChunk];
};
}  // namespace

// Pointers travel to the device as kernel arguments, 256 at a time: no pinned staging, nothing the
// call would have to keep alive, and the launch is an ordinary kernel node for a capturing caller.
__global__ void k_store_ptrs(uint64_t *dst, PtrChunk c, uint32_t n)
{
    if (threadIdx.x < n) dst[threadIdx.x] = c.p[threadIdx.x];
}

extern "C" int reft_parity_encode_noalloc(reft_plan *p, const void *const *shard_span_ptrs,
                                          uint32_t k, void *parity_dev, reft_stream stream)
{
    int rc = check_plan(p, "reft_parity_encode_noalloc");
    if (rc) return rc;
    if (k < 1 || k > REFT_MAX_K)
        return fail(REFT_EINVAL, "reft_parity_encode_noalloc: k = %u outside [1, %d]", k, REFT_MAX_K);
    const uint64_t n = (uint64_t)k * p->T;
    if (n > kScratchPtrs)
        return fail(REFT_ESIZE, "reft_parity_encode_noalloc: k * T = %llu span pointers, the static "
                                "scratch holds %u", (unsigned long long)n, kScratchPtrs);
    if ((rc = check_span_ptrs(p, shard_span_ptrs, k, "reft_parity_encode_noalloc"))) return rc;
    if (p->L == 0) return REFT_OK;
    if (!parity_dev) return fail(REFT_EINVAL, "reft_parity_encode_noalloc: null parity buffer");
    if (!p->scratch) return fail(REFT_EINVAL, "reft_parity_encode_noalloc: no static scratch on this GPU");
    hipStream_t s = (hipStream_t)stream;
    // p->scratch is the device address of `scratch` on the plan's GPU (hipGetSymbolAddress at plan
    // creation): the pointer table first, one block of burst counters behind it.  The table is
    // overwritten here and the counters are cleared by a kernel before each burst launch, so
    // nothing of an earlier call survives into this one.
    uint64_t *tab = (uint64_t *)p->scratch;
    uint32_t *ctr = (uint32_t *)(p->scratch + kScratchPtrBytes);
    for (uint64_t i = 0; i < n; i += kPtrChunk) {
        PtrChunk c;
        const uint32_t m = (uint32_t)(n - i < kPtrChunk ? n - i : kPtrChunk);
        for (uint32_t j = 0; j < m; ++j) c.p[j] = (uint64_t)(uintptr_t)shard_span_ptrs[i + j];
        for (uint32_t j = m; j < kPtrChunk; ++j) c.p[j] = 0;
        hipLaunchKernelGGL(k_store_ptrs, dim3(1), dim3(kPtrChunk), 0, s, tab + i, c, m);
        HIPCHK(hipGetLastError());
    }
    uint32_t next = 0;
    return xor_passes(p, tab, k, nullptr, nullptr, parity_dev, ctr, 1, &next, s);
}

// ------------------------------------------------------------------------------------------------
// rotated placement of the parity (section 4.2): every member protects one segment of every other
// ------------------------------------------------------------------------------------------------
namespace {
// One operand of a rotated XOR: the bytes at stream offsets [w, w + len) of a shard (bytes at or
// beyond L read as zero), or a contiguous buffer of len bytes.
struct WinSpec {
    bool contig;
    uint64_t w;
};
}  // namespace

static uint32_t rot_index(uint32_t i, uint32_t j) { return i < j ? i : i - 1; }

extern "C" uint64_t reft_segment_bytes(const reft_plan *p, uint32_t k)
{
    return (!p || k < 2) ? 0 : (p->L + (k - 2)) / (k - 1);
}

static int ensure_zeros(reft_plan *p)
{
    if (p->zeros) return REFT_OK;
    HIPCHK(hipMalloc(&p->zeros, 256));
    HIPCHK(hipMemset(p->zeros, 0, 256));
    return REFT_OK;
}

// The plan whose spans are the merged pieces of `nwin` windows of `len` bytes of the base plan
// (every span boundary of every window becomes a boundary), with the recipe that turns the
// caller's pointers into its rows.  Built on first use and kept in the base plan.
static int derived_plan(reft_plan *p, uint64_t key, const WinSpec *wins, uint32_t nwin, uint64_t len,
                        const DerivedPlan **out)
{
    auto it = p->derived.find(key);
    if (it != p->derived.end()) {
        *out = &it->second;
        return REFT_OK;
    }
    int rc = ensure_zeros(p);
    if (rc) return rc;
    std::vector<uint64_t> cuts{0, len};
    for (uint32_t q = 0; q < nwin; ++q) {
        if (wins[q].contig) continue;
        const uint64_t w = wins[q].w;
        // span starts strictly inside (w, w + len); off[T] = L makes the end of the stream a
        // boundary too, so the zero extension of the last segment starts on a piece boundary
        auto lo = std::upper_bound(p->off.begin(), p->off.end(), w);
        for (; lo != p->off.end() && *lo < w + len; ++lo) cuts.push_back(*lo - w);
    }
    std::sort(cuts.begin(), cuts.end());
    cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
    std::vector<uint64_t> sizes(cuts.size() - 1);
    for (size_t i = 0; i + 1 < cuts.size(); ++i) sizes[i] = cuts[i + 1] - cuts[i];
    DerivedPlan dp;
    if ((rc = reft_plan_create(sizes.data(), sizes.size(), nullptr, 0, 0, &dp.plan))) return rc;
    struct Guard {
        reft_plan *d;
        ~Guard() { if (d) reft_plan_destroy(d); }
    } guard{dp.plan};
    const reft_plan *d = dp.plan;
    dp.nwin = nwin;
    dp.recipe.resize((size_t)nwin * d->T);
    for (uint32_t q = 0; q < nwin; ++q)
        for (uint64_t t = 0; t < d->T; ++t) {
            RowRecipe &r = dp.recipe[(size_t)q * d->T + t];
            const uint64_t x = d->off[t];
            if (wins[q].contig) {
                r = RowRecipe{kContig, x};
                continue;
            }
            const uint64_t y = wins[q].w + x;
            if (y >= p->L) {                       // zero extension of the last segment
                if (d->off[t + 1] - x > 256) return fail(REFT_EINVAL, "internal: zero pad too long");
                r = RowRecipe{kZeros, 0};
                continue;
            }
            const uint64_t sp = (uint64_t)(std::upper_bound(p->off.begin(), p->off.end(), y) -
                                           p->off.begin()) - 1;        // off[sp] <= y < off[sp + 1]
            r = RowRecipe{(uint32_t)sp, y - p->off[sp]};
        }
    guard.d = nullptr;
    auto ins = p->derived.emplace(key, std::move(dp));
    *out = &ins.first->second;
    return REFT_OK;
}

// Row q of the derived plan's pointer table from the operand's own pointers.
static int window_row(const reft_plan *p, const DerivedPlan &dp, uint32_t q,
                      const void *const *span_ptrs, const void *contig, const void **row)
{
    const uint64_t Td = dp.plan->T;
    const RowRecipe *rec = dp.recipe.data() + (size_t)q * Td;
    for (uint64_t t = 0; t < Td; ++t) {
        if (rec[t].span == kContig) {
            row[t] = (const uint8_t *)contig + rec[t].add;
        } else if (rec[t].span == kZeros) {
            row[t] = p->zeros;
        } else {
            if (!span_ptrs[rec[t].span])
                return fail(REFT_EINVAL, "rotated parity: span %u is null but has bytes", rec[t].span);
            row[t] = (const uint8_t *)span_ptrs[rec[t].span] + rec[t].add;
        }
    }
    return REFT_OK;
}

extern "C" int reft_parity_encode_rotated(reft_plan *p, const void *const *shard_span_ptrs,
                                          uint32_t k, uint32_t member, void *parity_dev,
                                          reft_stream stream)
{
    REFT_GUARD_BEGIN
    int rc = check_plan(p, "reft_parity_encode_rotated");
    if (rc) return rc;
    if (k < 2 || k > REFT_MAX_K)
        return fail(REFT_EINVAL, "reft_parity_encode_rotated: k = %u outside [2, %d]", k, REFT_MAX_K);
    if (member >= k)
        return fail(REFT_EINVAL, "reft_parity_encode_rotated: member = %u but k = %u", member, k);
    if (!shard_span_ptrs) return fail(REFT_EINVAL, "reft_parity_encode_rotated: null pointer array");
    const uint64_t Lseg = reft_segment_bytes(p, k);
    if (Lseg == 0) return REFT_OK;
    if (!parity_dev) return fail(REFT_EINVAL, "reft_parity_encode_rotated: null parity buffer");
    WinSpec wins[REFT_MAX_K];
    uint32_t shard_of[REFT_MAX_K];
    uint32_t nwin = 0;
    for (uint32_t j = 0; j < k; ++j) {
        if (j == member) continue;
        shard_of[nwin] = j;
        wins[nwin++] = WinSpec{false, (uint64_t)rot_index(member, j) * Lseg};
    }
    const DerivedPlan *dp = nullptr;
    if ((rc = derived_plan(p, (1ull << 56) | ((uint64_t)k << 32) | member, wins, nwin, Lseg, &dp)))
        return rc;
    reft_plan *d = dp->plan;
    const void **rows = d->row_buf.data();
    for (uint32_t q = 0; q < nwin; ++q)
        if ((rc = window_row(p, *dp, q, shard_span_ptrs + (size_t)shard_of[q] * p->T, nullptr,
                             rows + (size_t)q * d->T)))
            return rc;
    return xor_rows(d, rows, nwin, nullptr, parity_dev, (hipStream_t)stream);
    REFT_GUARD_END("reft_parity_encode_rotated")
}

extern "C" int reft_reconstruct_rotated(reft_plan *p, const void *const *shard_span_ptrs,
                                        const void *const *parity_ptrs, uint32_t k, uint32_t lost,
                                        void *const *out_span_ptrs, reft_stream stream)
{
    REFT_GUARD_BEGIN
    int rc = check_plan(p, "reft_reconstruct_rotated");
    if (rc) return rc;
    if (k < 2 || k > REFT_MAX_K)
        return fail(REFT_EINVAL, "reft_reconstruct_rotated: k = %u outside [2, %d]", k, REFT_MAX_K);
    if (lost >= k) return fail(REFT_EINVAL, "reft_reconstruct_rotated: lost = %u but k = %u", lost, k);
    if (!shard_span_ptrs || !parity_ptrs)
        return fail(REFT_EINVAL, "reft_reconstruct_rotated: null pointer array");
    if ((rc = check_span_ptrs(p, out_span_ptrs, 1, "reft_reconstruct_rotated(out)"))) return rc;
    const uint64_t Lseg = reft_segment_bytes(p, k);
    if (Lseg == 0) return REFT_OK;
    for (uint32_t r = 0; r + 1 < k; ++r) {
        const uint64_t o0 = (uint64_t)r * Lseg;
        if (o0 >= p->L) break;
        const uint64_t len = p->L - o0 < Lseg ? p->L - o0 : Lseg;
        const uint32_t i = r < lost ? r : r + 1;          // the member that protects segment r
        if (!parity_ptrs[i])
            return fail(REFT_EINVAL, "reft_reconstruct_rotated: parity unit of member %u is null", i);
        // windows: the parity unit, the other segments it covers, and last the destination (its
        // own span boundaries must be piece boundaries too)
        WinSpec wins[REFT_MAX_K + 1];
        uint32_t shard_of[REFT_MAX_K + 1];
        uint32_t nwin = 0;
        shard_of[nwin] = 0;
        wins[nwin++] = WinSpec{true, 0};
        for (uint32_t j = 0; j < k; ++j) {
            if (j == i || j == lost) continue;
            shard_of[nwin] = j;
            wins[nwin++] = WinSpec{false, (uint64_t)rot_index(i, j) * Lseg};
        }
        shard_of[nwin] = lost;
        wins[nwin++] = WinSpec{false, o0};
        const DerivedPlan *dp = nullptr;
        if ((rc = derived_plan(p, (2ull << 56) | ((uint64_t)k << 32) | ((uint64_t)lost << 16) | r,
                               wins, nwin, len, &dp)))
            return rc;
        reft_plan *d = dp->plan;
        const void **rows = d->row_buf.data();
        if ((rc = window_row(p, *dp, 0, nullptr, parity_ptrs[i], rows))) return rc;
        for (uint32_t q = 1; q + 1 < nwin; ++q)
            if ((rc = window_row(p, *dp, q, shard_span_ptrs + (size_t)shard_of[q] * p->T, nullptr,
                                 rows + (size_t)q * d->T)))
                return rc;
        const void **dst = rows + (size_t)(nwin - 1) * d->T;      // where xor_rows wants it anyway
        if ((rc = window_row(p, *dp, nwin - 1, (const void *const *)out_span_ptrs, nullptr, dst)))
            return rc;
        if ((rc = xor_rows(d, rows, nwin - 1, dst, nullptr, (hipStream_t)stream))) return rc;
    }
    return REFT_OK;
    REFT_GUARD_END("reft_reconstruct_rotated")
}

// ------------------------------------------------------------------------------------------------
// several redundancy strategies at once (section 4.2): which lost members can be recovered, how
// ------------------------------------------------------------------------------------------------
extern "C" int reft_recovery_plan(uint32_t k, const uint32_t *copy_offsets, uint32_t n_copies,
                                  int parity_units, const uint8_t *lost, reft_recovery_step *steps,
                                  uint32_t *nsteps)
{
    if (!lost || !steps || !nsteps) return fail(REFT_EINVAL, "reft_recovery_plan: null argument");
    *nsteps = 0;
    if (k < 2 || k > REFT_MAX_K)
        return fail(REFT_EINVAL, "reft_recovery_plan: k = %u outside [2, %d]", k, REFT_MAX_K);
    if (n_copies && !copy_offsets) return fail(REFT_EINVAL, "reft_recovery_plan: null offsets");
    for (uint32_t a = 0; a < n_copies; ++a)
        if (copy_offsets[a] < 1 || copy_offsets[a] >= k)
            return fail(REFT_EINVAL, "reft_recovery_plan: copy offset %u outside [1, %u)",
                        copy_offsets[a], k);
    uint32_t nlost = 0, stuck = 0, first_stuck = 0;
    for (uint32_t x = 0; x < k; ++x) nlost += lost[x] ? 1u : 0u;
    for (uint32_t x = 0; x < k; ++x) {
        if (!lost[x]) continue;
        bool done = false;
        for (uint32_t a = 0; a < n_copies && !done; ++a) {
            const uint32_t holder = (x + k - copy_offsets[a]) % k;      // holder + d = x (mod k)
            if (lost[holder]) continue;
            steps[(*nsteps)++] = reft_recovery_step{x, REFT_RECOVER_COPY, holder, a};
            done = true;
        }
        // every segment of x is covered by the unit of another member: all of them must be there
        if (!done && parity_units && nlost == 1) {
            steps[(*nsteps)++] = reft_recovery_step{x, REFT_RECOVER_DECODE, 0, 0};
            done = true;
        }
        if (!done && stuck++ == 0) first_stuck = x;
    }
    if (stuck)
        return fail(REFT_EUNRECOVERABLE,
                    "reft_recovery_plan: %u of the %u lost members cannot be recovered (first: "
                    "member %u): no surviving duplicate%s", stuck, nlost, first_stuck,
                    parity_units ? ", and with more than one member lost a parity unit is missing too"
                                 : "");
    return REFT_OK;
}

// ------------------------------------------------------------------------------------------------
// S6: single-loss decode
// ------------------------------------------------------------------------------------------------
extern "C" int reft_reconstruct(const void *const *shards, uint32_t k, const void *parity,
                                uint64_t L, void *out_dev, uint32_t *lost_index,
                                reft_stream stream)
{
    REFT_GUARD_BEGIN
    if (!shards) return fail(REFT_EINVAL, "reft_reconstruct: null shard array");
    if (k < 1 || k > REFT_MAX_K - 1)
        return fail(REFT_EINVAL, "reft_reconstruct: k = %u outside [1, %d]", k, REFT_MAX_K - 1);
    uint32_t nlost = 0, lost = 0;
    for (uint32_t s = 0; s < k; ++s)
        if (!shards[s]) {
            if (nlost == 0) lost = s;
            ++nlost;
        }
    if (nlost >= 2)
        return fail(REFT_EUNRECOVERABLE,
                    "reft_reconstruct: %u of %u shards are lost; one parity decodes one loss",
                    nlost, k);
    if (nlost == 0) return fail(REFT_EINVAL, "reft_reconstruct: no shard is marked lost (NULL)");
    if (lost_index) *lost_index = lost;
    if (L == 0) return REFT_OK;
    if (!parity || !out_dev) return fail(REFT_EINVAL, "reft_reconstruct: null parity or output");

    uint64_t src[REFT_MAX_K];
    uint32_t n = 0;
    src[n++] = (uint64_t)(uintptr_t)parity;
    for (uint32_t s = 0; s < k; ++s)
        if (shards[s]) src[n++] = (uint64_t)(uintptr_t)shards[s];

    const LaunchCfg cfg = launch_cfg(nullptr);
    const uint32_t tile_shift = (uint32_t)g_tile_shift.load();
    hipStream_t st = (hipStream_t)stream;
    BurstCfg bc{};
    const bool burst_ok = g_burst.load() && L >= g_burst_min_bytes.load();
    uint32_t *ring = nullptr;
    int num_cus = 256;
    if (burst_ok) {
        // counter blocks from the ring in the library's static device memory (no allocation)
        const DeviceStatics *ds = nullptr;
        int rc = device_statics(&ds);
        if (rc) return rc;
        ring = ds->ctr;
        num_cus = ds->num_cus;
    }
    static std::atomic<uint32_t> next_slot{0};
    uint32_t done = 0;
    while (done < n) {
        SrcBases b{};
        int m = 0;
        if (done > 0) b.p[m++] = (uint64_t)(uintptr_t)out_dev;     // fold into the partial result
        while (m < kMaxSrc && done < n) b.p[m++] = src[done++];
        if (burst_ok && (uint32_t)m >= g_burst_min_rows.load()) {
            // reads and writes separated in time; folding in place is safe: a stage of the
            // output is read and, a round later, written by the same workgroup only
            bc = burst_cfg(ring, next_slot++ % kCtrBlocks, num_cus);
            HIPCHK(launch_xor_contig_burst(b, m, (uint64_t)(uintptr_t)out_dev, L, cfg, bc, st));
        } else {
            HIPCHK(launch_xor_contig(b, m, (uint64_t)(uintptr_t)out_dev, L, tile_shift, cfg, st));
        }
    }
    return REFT_OK;
    REFT_GUARD_END("reft_reconstruct")
}

// S6 + S7 in one pass: survivors read in place through their span tables, the parity as a
// contiguous stream, the result written straight into the lost shard's tensors.
extern "C" int reft_reconstruct_spans(reft_plan *p, const void *const *shard_span_ptrs, uint32_t k,
                                      uint32_t lost, const void *parity_dev,
                                      void *const *out_span_ptrs, reft_stream stream)
{
    REFT_GUARD_BEGIN
    int rc = check_plan(p, "reft_reconstruct_spans");
    if (rc) return rc;
    if (k < 1 || k > REFT_MAX_K - 1)
        return fail(REFT_EINVAL, "reft_reconstruct_spans: k = %u outside [1, %d]", k,
                    REFT_MAX_K - 1);
    if (lost >= k) return fail(REFT_EINVAL, "reft_reconstruct_spans: lost = %u but k = %u", lost, k);
    if (!shard_span_ptrs) return fail(REFT_EINVAL, "reft_reconstruct_spans: null pointer array");
    if ((rc = check_span_ptrs(p, out_span_ptrs, 1, "reft_reconstruct_spans(out)"))) return rc;
    // rows: the k-1 survivors, then the parity expressed as a span row
    const uint64_t T = p->T;
    const void **rows = p->row_buf.data();                     // (REFT_MAX_K + 1) * T entries
    uint32_t r = 0;
    for (uint32_t s = 0; s < k; ++s) {
        if (s == lost) continue;
        if ((rc = check_span_ptrs(p, shard_span_ptrs + (size_t)s * T, 1, "reft_reconstruct_spans")))
            return rc;
        for (uint64_t t = 0; t < T; ++t) rows[(size_t)r * T + t] = shard_span_ptrs[(size_t)s * T + t];
        ++r;
    }
    if (p->L == 0) return REFT_OK;
    if (!parity_dev) return fail(REFT_EINVAL, "reft_reconstruct_spans: null parity");
    for (uint64_t t = 0; t < T; ++t)
        rows[(size_t)r * T + t] = (const uint8_t *)parity_dev + p->off[t];
    ++r;                                                       // r == k source rows
    return xor_rows(p, rows, k, (const void *const *)out_span_ptrs, nullptr, (hipStream_t)stream);
    REFT_GUARD_END("reft_reconstruct_spans")
}

// ------------------------------------------------------------------------------------------------
// S5 + S7: restore
// ------------------------------------------------------------------------------------------------
extern "C" int reft_restore(reft_plan *p, const void *host_src, uint64_t host_bytes, void *staging,
                            uint64_t staging_bytes, void *const *span_ptrs,
                            reft_stream copy_stream, reft_stream unpack_stream)
{
    REFT_GUARD_BEGIN
    int rc = check_plan(p, "reft_restore");
    if (rc) return rc;
    if ((rc = check_span_ptrs(p, span_ptrs, 1, "reft_restore"))) return rc;
    if (host_bytes != p->L)
        return fail(REFT_ESIZE, "reft_restore: host snapshot has %llu bytes, stream has %llu",
                    (unsigned long long)host_bytes, (unsigned long long)p->L);
    if (p->L && !host_src) return fail(REFT_EINVAL, "reft_restore: null host buffer");
    hipStream_t cs = (hipStream_t)copy_stream, us = (hipStream_t)unpack_stream;
    const PlanTables pt = p->tables();
    const uint64_t *tab = nullptr;
    int entry = 0;

    if (!staging) {
        // Direct path: the scatter kernel loads the snapshot from pinned host memory itself.
        const uint64_t hview = p->L ? device_view_of_host(host_src) : 0;
        if (p->L && !hview)
            return fail(REFT_EINVAL, "reft_restore: host buffer is not mapped for device access "
                                     "(not pinned); pass a staging ring to copy it by DMA");
        if ((rc = upload_ptrs(p, span_ptrs, 1, us, &tab, &entry))) return rc;
        LaunchCfg cfg = link_cfg(p);
        cfg.max_wgs *= 2;          // reads across the link need about twice the waves of writes
        for (uint64_t b = 0; b < p->NB; ++b)
            HIPCHK(launch_scatter(pt, tab, hview, p->bstart[b], p->bstart[b + 1], cfg, us));
        if ((rc = release_ptrs(p, entry, us))) return rc;
        return record(p->rest_done, us);
    }

    int nslots = 1;
    if ((rc = staging_slots(p, staging, staging_bytes, "reft_restore", &nslots))) return rc;
    const PieceLists &pl = pieces_of(p, 0, p->NB);
    const std::vector<Run> &runs = pl.runs;
    const std::vector<Dma> &dmas = pl.dmas;
    const uint64_t stride = slot_stride(p);
    // The tensors are written on both streams.  The caller orders unpack_stream behind their last
    // use; copy_stream joins unpack_stream here so the same ordering covers its copies.
    if (us != cs) {
        if ((rc = record(p->rest_begin, us))) return rc;
        if ((rc = wait_on(cs, p->rest_begin))) return rc;
    }
    // large pieces: straight from the host snapshot into their tensors
    const uint64_t gmode = g_graph_copies.load();
    if (gmode && g_dma_streams.load() == 1 && dmas.size() >= 8) {
        if ((rc = copy_graph(p, dmas, cs, false, host_src, (const void *const *)span_ptrs, gmode)))
            return rc;
    } else if ((rc = issue_piece_copies(p, dmas, cs, [&](const Dma &d, hipStream_t st) {
                   return hipMemcpyAsync((uint8_t *)span_ptrs[d.span] + (d.o - p->off[d.span]),
                                         (const uint8_t *)host_src + d.o, d.n, hipMemcpyHostToDevice,
                                         st);
               })))
        return rc;
    if (!runs.empty()) {
        if ((rc = upload_ptrs(p, span_ptrs, 1, us, &tab, &entry))) return rc;
        const LaunchCfg cfg = launch_cfg(p);
        const int ngroups = nslots >= kGroups ? kGroups : 1;
        const uint64_t per_group = (uint64_t)(nslots / ngroups);
        uint64_t batch = 0;
        for (uint64_t r0 = 0; r0 < runs.size(); r0 += per_group, ++batch) {
            const int g = (int)(batch % (uint64_t)ngroups);
            const uint64_t r1 = r0 + per_group < runs.size() ? r0 + per_group : runs.size();
            // the group's previous occupants must have been scattered
            if ((rc = wait_on(cs, p->rest_free[g]))) return rc;
            for (uint64_t r = r0; r < r1; ++r) {
                const uint64_t slot = (uint64_t)g * per_group + (r - r0);
                const uint64_t slot_addr =
                    (uint64_t)(uintptr_t)staging + slot * stride + (runs[r].a & 255);
                HIPCHK(hipMemcpyAsync((void *)(uintptr_t)slot_addr,
                                      (const uint8_t *)host_src + runs[r].a, runs[r].b - runs[r].a,
                                      hipMemcpyHostToDevice, cs));
            }
            if ((rc = record(p->rest_filled[g], cs))) return rc;
            if ((rc = wait_on(us, p->rest_filled[g]))) return rc;
            for (uint64_t r = r0; r < r1; ++r) {
                const uint64_t slot = (uint64_t)g * per_group + (r - r0);
                const uint64_t slot_addr =
                    (uint64_t)(uintptr_t)staging + slot * stride + (runs[r].a & 255);
                HIPCHK(launch_scatter(pt, tab, slot_addr - runs[r].a, runs[r].a, runs[r].b, cfg, us));
            }
            if ((rc = record(p->rest_free[g], us))) return rc;
        }
        if ((rc = release_ptrs(p, entry, us))) return rc;
    }
    // completion on unpack_stream: behind the scatter kernels and behind every direct copy
    if ((rc = record(p->rest_copied, cs))) return rc;
    if ((rc = wait_on(us, p->rest_copied))) return rc;
    return record(p->rest_done, us);
    REFT_GUARD_END("reft_restore")
}

extern "C" int reft_restore_wait(reft_plan *p)
{
    int rc = check_plan(p, "reft_restore_wait");
    if (rc) return rc;
    if (p->rest_done.recorded) HIPCHK(hipEventSynchronize(p->rest_done.ev));
    return REFT_OK;
}
