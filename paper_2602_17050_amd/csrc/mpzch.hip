// Host side of the C ABI declared in include/mpzch.h: argument checks, scratch management and
// kernel launches on the caller's stream.  No call here synchronises with the host except
// where the header says so (scratch growth, descriptor upload, timing read-out, destroy).
#include "../../include/mpzch.h"
#include "mpzch_kernels.hpp"

#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace mpzch;

namespace {

struct TableCfg {
    int64_t num_slots;
    int32_t max_probe;
    int32_t kind;
    int32_t ttl;
    uint64_t seed;
    int32_t layout;                // MPZCH_LAYOUT_*
};

// ---- per-kernel timing --------------------------------------------------------------------
enum KernelId { KDiscover = 0, KAllocate, KFinalize, KLookup, KernelCount };
const char *const kKernelNames[KernelCount] = {"k_discover", "k_allocate", "k_finalize", "k_lookup"};

struct Timing {
    bool enabled = false;
    bool pass1_only = false;       // bracket k_discover / k_lookup only (two events per call instead of eight)
    int every = 1;                 // ... and of those launches only every `every`-th
    int64_t pass1_seen = 0;
    bool skipped = false;          // the launch between the last begin and end is not bracketed
    void set_mode(int32_t enable)
    {
        enabled = enable != 0;
        pass1_only = enable == 2 || enable == 3;
        every = enable == 3 ? 4 : 1;
        pass1_seen = 0;
    }
    struct Rec { int kernel; hipEvent_t a, b; };
    std::vector<Rec> used;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;

    bool begin(int kernel, hipStream_t s)
    {
        skipped = !enabled || (pass1_only && kernel != KDiscover && kernel != KLookup);
        if (!skipped && pass1_only) skipped = (pass1_seen++ % every) != every - 1;
        if (skipped) return true;
        std::pair<hipEvent_t, hipEvent_t> ev;
        if (!pool.empty()) {
            ev = pool.back();
            pool.pop_back();
        } else {
            if (hipEventCreate(&ev.first) != hipSuccess) return false;
            if (hipEventCreate(&ev.second) != hipSuccess) { (void)hipEventDestroy(ev.first); return false; }
        }
        used.push_back({kernel, ev.first, ev.second});
        return hipEventRecord(ev.first, s) == hipSuccess;
    }
    bool end(hipStream_t s)
    {
        if (skipped) return true;
        return hipEventRecord(used.back().b, s) == hipSuccess;
    }
    mpzch_status_t collect(const char **names, double *ms, int64_t *launches, int32_t cap, int32_t *count)
    {
        double acc[KernelCount] = {0};
        int64_t cnt[KernelCount] = {0};
        for (auto &r : used) {
            if (hipEventSynchronize(r.b) != hipSuccess) return MPZCH_ERR_HIP;
            float t = 0.f;
            if (hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) return MPZCH_ERR_HIP;
            acc[r.kernel] += t;
            cnt[r.kernel]++;
            pool.push_back({r.a, r.b});
        }
        used.clear();
        int32_t k = 0;
        for (int i = 0; i < KernelCount && k < cap; ++i) {
            if (!cnt[i]) continue;
            names[k] = kKernelNames[i];
            ms[k] = acc[i];
            launches[k] = cnt[i];
            ++k;
        }
        *count = k;
        return MPZCH_OK;
    }
    void destroy()
    {
        for (auto &r : used) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (auto &e : pool) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
        used.clear();
        pool.clear();
    }
};

// ---- device scratch -----------------------------------------------------------------------
// Grid caps in workgroups per compute unit.  8 is the measured best for Pass 1 (4 and 16 are within a few
// per cent) and for the kernels that walk the miss lists; scratch is sized for up to kDiscoverBlocksPerCuMax.
const int kDiscoverBlocksPerCuMax = 16;
constexpr int discover_blocks_per_cu() { return 8; }
constexpr int group_blocks_per_cu() { return 8; }

// Compute units of the current device, asked once per device and process (no handle state: read-only
// entry points take const handles).
mpzch_status_t device_cus(int *out)
{
    static std::mutex mu;
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MPZCH_ERR_HIP;
    if (dev < 0 || dev >= 64) return MPZCH_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!cus[dev]) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return MPZCH_ERR_HIP;
        cus[dev] = n;
    }
    *out = cus[dev];
    return MPZCH_OK;
}

struct Scratch {
    char *base = nullptr;
    int64_t cap_n = 0;
    uint32_t *list = nullptr;
    uint32_t *ent = nullptr;
    uint32_t *first_of = nullptr;
    int64_t *homes = nullptr;
    uint8_t *hint = nullptr;
    uint32_t *seg_cnt = nullptr;
    uint32_t *set_slot = nullptr;
    Control *ctl = nullptr;
    Control *lookup_ctl = nullptr; // counter block of counting lookups while there is no scratch area
    bool dirty = false;            // a launch sequence was cut short: set and counters must be cleared before use
    bool owned = true;             // base came from hipMalloc (false: it points into the file-scope scratch array)
    int num_cus = 0;

    static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

    mpzch_status_t query_device()
    {
        if (num_cus) return MPZCH_OK;
        return device_cus(&num_cus);
    }

    // Where each array sits inside an area that serves batches of up to n positions: 29 bytes per
    // position and a few small fixed areas.
    struct Layout {
        size_t o_list, o_ent, o_first, o_homes, o_hint, o_seg, o_set, o_ctl, total;
    };
    static Layout layout_for(int64_t n, int num_cus)
    {
        Layout L;
        const size_t max_blocks = (size_t)num_cus * kDiscoverBlocksPerCuMax;
        const size_t per_pos = 4 * ((size_t)n + 2 * kWave);   // list-shaped arrays: n + 128 entries
        L.o_list = 0;
        L.o_ent = L.o_list + align_up(per_pos);
        L.o_first = L.o_ent + align_up(per_pos);
        L.o_homes = L.o_first + align_up(per_pos);
        L.o_hint = L.o_homes + align_up(2 * per_pos);
        L.o_seg = L.o_hint + align_up((size_t)n + kWave);
        L.o_set = L.o_seg + align_up(4 * max_blocks * kWavesPerBlock);
        L.o_ctl = L.o_set + align_up(8 * (size_t)n);
        L.total = L.o_ctl + align_up(sizeof(Control));
        return L;
    }
    void bind(char *area, const Layout &L, int64_t n)
    {
        base = area;
        list = (uint32_t *)(base + L.o_list);
        ent = (uint32_t *)(base + L.o_ent);
        first_of = (uint32_t *)(base + L.o_first);
        homes = (int64_t *)(base + L.o_homes);
        hint = (uint8_t *)(base + L.o_hint);
        seg_cnt = (uint32_t *)(base + L.o_seg);
        set_slot = (uint32_t *)(base + L.o_set);
        ctl = (Control *)(base + L.o_ctl);
        cap_n = n;
    }

    mpzch_status_t ensure(int64_t n)
    {
        mpzch_status_t st = query_device();
        if (st != MPZCH_OK) return st;
        if (n <= cap_n && base) return MPZCH_OK;
        if (n < 1024) n = 1024;
        if (base) {
            if (hipDeviceSynchronize() != hipSuccess) return MPZCH_ERR_HIP;
            (void)hipFree(base);
            base = nullptr;
            cap_n = 0;
        }
        const Layout L = layout_for(n, num_cus);
        char *area = nullptr;
        if (hipMalloc((void **)&area, L.total) != hipSuccess) return MPZCH_ERR_ALLOC;
        bind(area, L, 0);
        // empty set (0xFFFFFFFF) and zero counters; set entries are re-emptied by every call, so
        // this is the only full clear
        if (hipMemset(base + L.o_set, 0xFF, (L.o_ctl - L.o_set)) != hipSuccess) return MPZCH_ERR_HIP;
        if (hipMemset(base + L.o_ctl, 0, L.total - L.o_ctl) != hipSuccess) return MPZCH_ERR_HIP;
        if (hipDeviceSynchronize() != hipSuccess) return MPZCH_ERR_HIP;
        cap_n = n;
        return MPZCH_OK;
    }
    // the counter block alone (a counting lookup needs nothing else): the scratch area's when there is one
    mpzch_status_t ensure_ctl(Control **out)
    {
        if (base) { *out = ctl; return MPZCH_OK; }
        if (!lookup_ctl) {
            if (hipMalloc((void **)&lookup_ctl, sizeof(Control)) != hipSuccess) { lookup_ctl = nullptr; return MPZCH_ERR_ALLOC; }
            if (hipMemset(lookup_ctl, 0, sizeof(Control)) != hipSuccess) return MPZCH_ERR_HIP;
            if (hipDeviceSynchronize() != hipSuccess) return MPZCH_ERR_HIP;
        }
        *out = lookup_ctl;
        return MPZCH_OK;
    }
    void release()
    {
        if (base && owned) { (void)hipDeviceSynchronize(); (void)hipFree(base); }
        if (lookup_ctl) { (void)hipDeviceSynchronize(); (void)hipFree(lookup_ctl); lookup_ctl = nullptr; }
        base = nullptr;
        cap_n = 0;
    }
};

int grid_for(int64_t items, int64_t items_per_block, int num_cus, int blocks_per_cu)
{
    int64_t b = (items + items_per_block - 1) / items_per_block;
    const int64_t cap = (int64_t)num_cus * blocks_per_cu;
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

static_assert(kLruLongProbe == MPZCH_MAX_PROBE_LRU, "the LRU kernels hold max_probe / 64 slots per lane");

int32_t p_eff(const TableCfg &c) { return (int64_t)c.max_probe < c.num_slots ? c.max_probe : (int32_t)c.num_slots; }

TableDesc make_desc(const TableCfg &c, int64_t *I, int32_t *M, int64_t ev_begin, int64_t ev_cap)
{
    TableDesc d;
    d.I = I;
    d.M = M;
    d.N = c.num_slots;
    d.seed = c.seed;
    d.P = p_eff(c);
    d.ttl = c.ttl;
    d.evict = c.kind == MPZCH_EVICT_TTL ? 1 : c.kind == MPZCH_EVICT_LRU ? 2 : c.kind == MPZCH_EVICT_TTL_EXPIRY ? 3 : 0;
    d.sh = c.layout == MPZCH_LAYOUT_RECORDS ? 1 : 0;
    d.ev_begin = ev_begin;
    d.ev_cap = ev_cap;
    return d;
}

#define LAUNCH_CHECK()                                        \
    do {                                                      \
        if (hipGetLastError() != hipSuccess) return MPZCH_ERR_HIP; \
    } while (0)

// two-tensor tables from this size on (1 GiB of identities, four times the memory-side cache) are probed with
// non-temporal loads in training
constexpr int64_t kStreamingSlots = (int64_t)1 << 27;

template <bool TRAIN>
mpzch_status_t launch_discover(const Params &p, int grid, hipStream_t s)
{
    if (TRAIN) {
        if (p.num_tables > 1) hipLaunchKernelGGL(k_discover_tables, dim3(grid), dim3(kBlock), 0, s, p);
        else if (p.t0.sh) hipLaunchKernelGGL(k_discover_records, dim3(grid), dim3(kBlock), 0, s, p);
        else if (p.t0.N >= kStreamingSlots) hipLaunchKernelGGL(k_discover_streaming, dim3(grid), dim3(kBlock), 0, s, p);
        else hipLaunchKernelGGL(k_discover, dim3(grid), dim3(kBlock), 0, s, p);
    } else {
        if (p.num_tables > 1) hipLaunchKernelGGL(k_lookup_tables, dim3(grid), dim3(kBlock), 0, s, p);
        else hipLaunchKernelGGL(k_lookup, dim3(grid), dim3(kBlock), 0, s, p);
    }
    LAUNCH_CHECK();
    return MPZCH_OK;
}

// max_p: largest min(max_probe, num_slots) of the tables involved; max_p_lru: the same over the LRU
// tables, 0 when there is none
template <bool MULTI>
void launch_allocate_lru(int32_t max_p_lru, const Params &p, int grid, hipStream_t s)
{
    // a group of 8, 16, 32 or 64 lanes per claimant, whichever holds its window; the whole wavefront
    // with several slots per lane for longer probe ranges
    if (max_p_lru > kWave) hipLaunchKernelGGL((k_allocate_lru_long<MULTI>), dim3(grid), dim3(kWave), 0, s, p);
    else if (max_p_lru <= 8) hipLaunchKernelGGL((k_allocate_lru<8, MULTI>), dim3(grid), dim3(kWave), 0, s, p);
    else if (max_p_lru <= 16) hipLaunchKernelGGL((k_allocate_lru<16, MULTI>), dim3(grid), dim3(kWave), 0, s, p);
    else if (max_p_lru <= 32) hipLaunchKernelGGL((k_allocate_lru<32, MULTI>), dim3(grid), dim3(kWave), 0, s, p);
    else hipLaunchKernelGGL((k_allocate_lru<64, MULTI>), dim3(grid), dim3(kWave), 0, s, p);
}

mpzch_status_t launch_allocate(int32_t max_p, int32_t max_p_lru, const Params &p, int num_cus, hipStream_t s)
{
    // one wavefront per workgroup, one segment per workgroup pass; the lane phase covers the first
    // 8 or 16 slots of every window, longer windows continue in the wave phase
    const int grid = grid_for((int64_t)p.num_segs, 1, num_cus, 4 * group_blocks_per_cu());
    if (p.num_tables > 1) {
        // several tables: TTL / no-eviction claimants first (this also writes every hint), then
        // the claimants of LRU tables
        if (max_p <= 8) hipLaunchKernelGGL((k_allocate<8, true>), dim3(grid), dim3(kWave), 0, s, p);
        else hipLaunchKernelGGL((k_allocate<16, true>), dim3(grid), dim3(kWave), 0, s, p);
        LAUNCH_CHECK();
        if (max_p_lru > 0) launch_allocate_lru<true>(max_p_lru, p, grid, s);
    } else if (max_p_lru > 0) {
        launch_allocate_lru<false>(max_p_lru, p, grid, s);
    } else {
        if (max_p <= 8) hipLaunchKernelGGL((k_allocate<8, false>), dim3(grid), dim3(kWave), 0, s, p);
        else hipLaunchKernelGGL((k_allocate<16, false>), dim3(grid), dim3(kWave), 0, s, p);
    }
    LAUNCH_CHECK();
    return MPZCH_OK;
}

mpzch_status_t launch_finalize(const Params &p, int grid, hipStream_t s)
{
    hipLaunchKernelGGL(k_finalize, dim3(grid), dim3(kBlock), 0, s, p);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

#define TRY(expr)                                   \
    do {                                            \
        mpzch_status_t st__ = (expr);               \
        if (st__ != MPZCH_OK) return st__;          \
    } while (0)
#define TIMED(tm, id, s, launch)                    \
    do {                                            \
        if (!(tm).begin((id), (s))) return MPZCH_ERR_HIP; \
        TRY(launch);                                \
        if (!(tm).end((s))) return MPZCH_ERR_HIP;   \
    } while (0)

mpzch_status_t fill64(int64_t *dst, int64_t count, long long value, hipStream_t s);
mpzch_status_t fill32(int32_t *dst, int64_t count, int32_t value, hipStream_t s);

// The launch sequence of one training remap (single table or group).
mpzch_status_t launch_remap(Scratch &sc, Timing &tm, Params p, int32_t max_p, int32_t max_p_lru, hipStream_t s);

// Every call leaves the scratch set empty and the counter block zeroed -- unless its launch
// sequence was cut short by a HIP error; the next call then clears both before it starts.
mpzch_status_t run_remap(Scratch &sc, Timing &tm, const Params &p, int32_t max_p, int32_t max_p_lru, hipStream_t s)
{
    if (sc.dirty) {
        TRY(fill32((int32_t *)sc.set_slot, 2 * sc.cap_n, -1, s));
        TRY(fill64((int64_t *)sc.ctl, (int64_t)(sizeof(Control) / sizeof(int64_t)), 0, s));
    }
    sc.dirty = true;
    const mpzch_status_t st = launch_remap(sc, tm, p, max_p, max_p_lru, s);
    if (st == MPZCH_OK) sc.dirty = false;
    return st;
}

mpzch_status_t launch_remap(Scratch &sc, Timing &tm, Params p, int32_t max_p, int32_t max_p_lru, hipStream_t s)
{
    p.list = sc.list;
    p.ent = sc.ent;
    p.first_of = sc.first_of;
    p.hint = sc.hint;
    p.homes = sc.homes;
    p.seg_cnt = sc.seg_cnt;
    p.set_slot = sc.set_slot;
    p.ctl = sc.ctl;

    const int64_t num_chunks = (p.n + kWave - 1) / kWave;
    // k_discover: every wavefront owns one segment of seg_chunks 64-position chunks
    const int g_disc = grid_for(p.n, kBlock, sc.num_cus, discover_blocks_per_cu());
    p.num_segs = g_disc * kWavesPerBlock;
    p.seg_chunks = (int32_t)((num_chunks + p.num_segs - 1) / p.num_segs);
    // the other kernels walk the segments' miss lists, one segment per wavefront pass
    const int g_grp = grid_for((int64_t)p.num_segs, kWavesPerBlock, sc.num_cus, group_blocks_per_cu());

    TIMED(tm, KDiscover, s, (launch_discover<true>(p, g_disc, s)));
    TIMED(tm, KAllocate, s, launch_allocate(max_p, max_p_lru, p, sc.num_cus, s));
    TIMED(tm, KFinalize, s, launch_finalize(p, g_grp, s));
    return MPZCH_OK;
}

mpzch_status_t fill64(int64_t *dst, int64_t count, long long value, hipStream_t s)
{
    if (count <= 0) return MPZCH_OK;
    const int grid = (int)((count + kBlock - 1) / kBlock < 4096 ? (count + kBlock - 1) / kBlock : 4096);
    hipLaunchKernelGGL(k_fill64, dim3(grid), dim3(kBlock), 0, s, (long long *)dst, count, value);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

mpzch_status_t fill32(int32_t *dst, int64_t count, int32_t value, hipStream_t s)
{
    if (count <= 0) return MPZCH_OK;
    const int grid = (int)((count + kBlock - 1) / kBlock < 4096 ? (count + kBlock - 1) / kBlock : 4096);
    hipLaunchKernelGGL(k_fill32, dim3(grid), dim3(kBlock), 0, s, dst, count, value);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

// one tensor of 16-byte records: identities points at record 0 (16-byte aligned), metadata at its third word
bool records_ok(const int64_t *identities, const int32_t *metadata)
{
    return !((uintptr_t)identities & 15) && (const void *)metadata == (const void *)((const int32_t *)identities + 2);
}
// the kernels keep the address of a slot in 48 bits (device addresses have no more)
bool addresses_ok(const TableCfg &c, const int64_t *identities)
{
    const uint64_t bytes = (uint64_t)c.num_slots << (c.layout == MPZCH_LAYOUT_RECORDS ? 4 : 3);
    const uint64_t begin = (uint64_t)(uintptr_t)identities;
    return identities && !(begin >> 48) && !((begin + bytes) >> 48);
}
bool layout_ok(const TableCfg &c, const int64_t *identities, const int32_t *metadata)
{
    return addresses_ok(c, identities) && (c.layout != MPZCH_LAYOUT_RECORDS || records_ok(identities, metadata));
}
// the read-only entry points see the identities only: records start at a multiple of 16 bytes
bool identities_ok(const TableCfg &c, const int64_t *identities)
{
    return addresses_ok(c, identities) && (c.layout != MPZCH_LAYOUT_RECORDS || !((uintptr_t)identities & 15));
}

bool valid_cfg(int64_t num_slots, int32_t max_probe, mpzch_eviction_policy_t policy)
{
    if (num_slots < 1 || num_slots > MPZCH_MAX_SLOTS || max_probe < 1 || max_probe > MPZCH_MAX_PROBE) return false;
    if (policy.kind != MPZCH_EVICT_NONE && policy.kind != MPZCH_EVICT_TTL && policy.kind != MPZCH_EVICT_LRU &&
        policy.kind != MPZCH_EVICT_TTL_EXPIRY)
        return false;
    if (policy.ttl < 0) return false;
    return true;
}

}  // namespace

// ---- the entry point that allocates nothing ------------------------------------------------------
// Its scratch is this file-scope array in device memory (every GPU the library runs on holds its own
// copy until the process ends).  In host code the array's name is only a handle for
// hipGetSymbolAddress: the address that kernels and fills receive is the one that call returns,
// queried once per device and kept in g_static.
constexpr size_t kStaticScratchBytes = (size_t)MPZCH_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
struct StaticState {
    bool ready = false;
    Scratch sc;
};
StaticState g_static[kMaxDevices];
std::mutex g_static_mutex;

// Set-up on the current device (first call on it): the array's address on this device, the layout of
// the scratch arrays inside it, and the one full clear (empty set, zero counters).
mpzch_status_t static_scratch(hipStream_t s, Scratch **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MPZCH_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return MPZCH_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticState &st = g_static[dev];
    if (!st.ready) {
        TRY(st.sc.query_device());
        const Scratch::Layout L = Scratch::layout_for(MPZCH_NOALLOC_MAX_BATCH, st.sc.num_cus);
        if (L.total > kStaticScratchBytes) return MPZCH_ERR_UNSUPPORTED;     // a GPU with far more compute units
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MPZCH_ERR_HIP;
        st.sc.owned = false;
        st.sc.bind((char *)ptr, L, MPZCH_NOALLOC_MAX_BATCH);
        // fill kernels, not memsets: the first call may sit in a stream whose work a caller replays
        TRY(fill32((int32_t *)st.sc.set_slot, (int64_t)((L.o_ctl - L.o_set) / 4), -1, s));
        TRY(fill64((int64_t *)(st.sc.base + L.o_ctl), (int64_t)((L.total - L.o_ctl) / 8), 0, s));
        st.ready = true;
    }
    *out = &st.sc;
    return MPZCH_OK;
}
}  // namespace

struct mpzch_table {
    TableCfg cfg;
    Scratch sc;
    mutable Timing tm;             // benchmark instrumentation: also records the launches of read-only calls
};

// A device copy of per-table descriptors of a group, re-uploaded only when one of them changes.
template <typename D>
struct DevCache {
    D *dev = nullptr;
    std::vector<D> host;                 // what dev holds
    bool uploaded = false;

    mpzch_status_t put(const std::vector<D> &descs, hipStream_t s)
    {
        if (!dev && hipMalloc((void **)&dev, sizeof(D) * MPZCH_MAX_GROUP_TABLES) != hipSuccess) {
            dev = nullptr;
            return MPZCH_ERR_ALLOC;
        }
        const size_t bytes = sizeof(D) * descs.size();
        if (!uploaded || host.size() != descs.size() || std::memcmp(host.data(), descs.data(), bytes) != 0) {
            // earlier calls on this stream may still read the old descriptors
            if (hipStreamSynchronize(s) != hipSuccess) return MPZCH_ERR_HIP;
            if (hipMemcpy(dev, descs.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return MPZCH_ERR_HIP;
            host = descs;
            uploaded = true;
        }
        return MPZCH_OK;
    }
    void release()
    {
        if (dev) (void)hipFree(dev);
        dev = nullptr;
        uploaded = false;
    }
};

struct mpzch_group {
    std::vector<TableCfg> cfgs;
    Scratch sc;
    Timing tm;
    DevCache<TableDesc> train;           // descriptors of mpzch_remap_jagged (identities + metadata)
    DevCache<TableDesc> infer;           // descriptors of mpzch_lookup_jagged (identities only)
    DevCache<JagRows> rows;              // descriptors of mpzch_reset_rows_jagged
};

extern "C" {

mpzch_status_t mpzch_create(int64_t num_slots, int32_t max_probe, mpzch_eviction_policy_t policy,
                            uint64_t hash_seed, mpzch_table_t **out)
{
    return mpzch_create_with_layout(num_slots, max_probe, policy, hash_seed, MPZCH_LAYOUT_SEPARATE, out);
}

mpzch_status_t mpzch_create_with_layout(int64_t num_slots, int32_t max_probe, mpzch_eviction_policy_t policy,
                                        uint64_t hash_seed, int32_t layout, mpzch_table_t **out)
{
    if (!out) return MPZCH_ERR_INVALID_ARG;
    *out = nullptr;
    if (layout != MPZCH_LAYOUT_SEPARATE && layout != MPZCH_LAYOUT_RECORDS) return MPZCH_ERR_INVALID_ARG;
    if (!valid_cfg(num_slots, max_probe, policy)) return MPZCH_ERR_INVALID_ARG;
    if (policy.kind == MPZCH_EVICT_LRU && max_probe > MPZCH_MAX_PROBE_LRU) return MPZCH_ERR_UNSUPPORTED;
    mpzch_table *t = new (std::nothrow) mpzch_table();
    if (!t) return MPZCH_ERR_ALLOC;
    t->cfg = {num_slots, max_probe, policy.kind, policy.ttl, hash_seed, layout};
    *out = t;
    return MPZCH_OK;
}

mpzch_status_t mpzch_destroy(mpzch_table_t *t)
{
    if (!t) return MPZCH_OK;
    t->sc.release();
    t->tm.destroy();
    delete t;
    return MPZCH_OK;
}

mpzch_status_t mpzch_reserve(mpzch_table_t *t, int64_t max_n)
{
    if (!t || max_n < 0 || max_n > MPZCH_MAX_BATCH) return MPZCH_ERR_INVALID_ARG;
    return t->sc.ensure(max_n);
}

mpzch_status_t mpzch_init_tensors(const mpzch_table_t *t, int64_t *identities, int32_t *metadata, void *stream)
{
    if (!t || !identities) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (t->cfg.layout == MPZCH_LAYOUT_RECORDS) {
        if (!records_ok(identities, metadata)) return MPZCH_ERR_INVALID_ARG;
        const int64_t count = t->cfg.num_slots;
        const int grid = (int)((count + kBlock - 1) / kBlock < 4096 ? (count + kBlock - 1) / kBlock : 4096);
        hipLaunchKernelGGL(k_init_records, dim3(grid), dim3(kBlock), 0, s, (u32x4 *)identities, count);
        LAUNCH_CHECK();
        return MPZCH_OK;
    }
    TRY(fill64(identities, t->cfg.num_slots, -1, s));
    if (metadata) TRY(fill32(metadata, t->cfg.num_slots, -1, s));
    return MPZCH_OK;
}

namespace {
// geometry shared by the row movers: 16-byte chunks when everything is 16-byte aligned, else 4-byte
struct RowGeom { bool ok; bool wide; int64_t chunks; };
RowGeom row_geom(const void *rows, int64_t row_bytes, int64_t row_stride_bytes, const void *other)
{
    RowGeom g{false, false, 0};
    if (row_bytes < 4 || row_stride_bytes < row_bytes || (row_bytes & 3) || (row_stride_bytes & 3)) return g;
    if (((uintptr_t)rows & 3) || ((uintptr_t)other & 3)) return g;
    g.wide = !(row_bytes & 15) && !(row_stride_bytes & 15) && !((uintptr_t)rows & 15) && !((uintptr_t)other & 15);
    g.chunks = g.wide ? row_bytes / 16 : row_bytes / 4;
    g.ok = g.chunks <= 0x7FFFFFFF;
    return g;
}
int row_grid(int64_t items)
{
    int64_t want = (items + kBlock - 1) / kBlock;
    if (want > 8192) want = 8192;
    if (want < 1) want = 1;
    return (int)want;
}
}  // namespace

namespace {
// rows that a remap resets itself (mpzch_remap_reset), or none
struct ResetRows {
    void *rows = nullptr;
    int64_t num_rows = 0, row_bytes = 0, row_stride_bytes = 0;
    const void *init_row = nullptr;
};

mpzch_status_t remap_one(mpzch_table_t *t, int64_t *identities, int32_t *metadata, const int64_t *ids,
                         const int32_t *ttls, int64_t n, int32_t step, int64_t *out_slots,
                         int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                         int64_t *out_stats, const ResetRows &rr, void *stream)
{
    if (!t || !identities || !metadata || !out_num_evicted) return MPZCH_ERR_INVALID_ARG;
    if (n < 0 || n > MPZCH_MAX_BATCH || step < 0 || evicted_cap < 0) return MPZCH_ERR_INVALID_ARG;
    if (ttls && t->cfg.kind != MPZCH_EVICT_TTL_EXPIRY) return MPZCH_ERR_INVALID_ARG;
    if (!layout_ok(t->cfg, identities, metadata)) return MPZCH_ERR_INVALID_ARG;
    if (n > 0 && (!ids || !out_slots)) return MPZCH_ERR_INVALID_ARG;
    if (evicted_cap > 0 && !out_evicted_slots) return MPZCH_ERR_INVALID_ARG;
    RowGeom g{true, false, 0};
    if (rr.rows) {
        if (rr.num_rows < 1) return MPZCH_ERR_INVALID_ARG;
        g = row_geom(rr.rows, rr.row_bytes, rr.row_stride_bytes, rr.init_row);
        if (!g.ok) return MPZCH_ERR_INVALID_ARG;
    }
    hipStream_t s = (hipStream_t)stream;
    if (n == 0) {
        TRY(fill64(out_num_evicted, 1, 0, s));
        if (out_stats) TRY(fill64(out_stats, MPZCH_STAT_COUNT, 0, s));
        return MPZCH_OK;
    }
    TRY(t->sc.ensure(n));
    Params p;
    std::memset(&p, 0, sizeof p);
    p.ids = ids;
    p.ttls = ttls;
    p.n = n;
    p.step = step;
    p.num_tables = 1;
    p.out_slots = out_slots;
    p.t0 = make_desc(t->cfg, identities, metadata, 0, evicted_cap);
    p.out_evicted = out_evicted_slots;
    p.out_num_evicted = out_num_evicted;
    p.out_stats = out_stats;
    if (rr.rows) {
        p.r_rows = (char *)rr.rows;
        p.r_init = rr.init_row;
        p.g_num_rows = rr.num_rows;
        p.g_stride = rr.row_stride_bytes;
        p.g_chunks = (int32_t)g.chunks;
        p.g_wide = g.wide ? 1 : 0;
        p.g_shift = -1;
        for (int b = 0; b < 31; ++b)
            if (g.chunks == ((int64_t)1 << b)) p.g_shift = b;
    }
    return run_remap(t->sc, t->tm, p, p.t0.P, p.t0.evict == 2 ? p.t0.P : 0, s);
}
}  // namespace

mpzch_status_t mpzch_remap_feature_ttl(mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                                       const int64_t *ids, const int32_t *ttls, int64_t n, int32_t step,
                                       int64_t *out_slots,
                                       int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                                       int64_t *out_stats, void *stream)
{
    return remap_one(t, identities, metadata, ids, ttls, n, step, out_slots, out_evicted_slots, evicted_cap,
                     out_num_evicted, out_stats, ResetRows{}, stream);
}

mpzch_status_t mpzch_remap(mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                           const int64_t *ids, int64_t n, int32_t step,
                           int64_t *out_slots,
                           int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                           int64_t *out_stats, void *stream)
{
    return remap_one(t, identities, metadata, ids, nullptr, n, step, out_slots, out_evicted_slots, evicted_cap,
                     out_num_evicted, out_stats, ResetRows{}, stream);
}

mpzch_status_t mpzch_remap_reset(mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                                 const int64_t *ids, int64_t n, int32_t step,
                                 int64_t *out_slots,
                                 int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                                 int64_t *out_stats,
                                 void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                 const void *init_row, void *stream)
{
    if (!rows) return MPZCH_ERR_INVALID_ARG;
    ResetRows rr;
    rr.rows = rows;
    rr.num_rows = num_rows;
    rr.row_bytes = row_bytes;
    rr.row_stride_bytes = row_stride_bytes;
    rr.init_row = init_row;
    return remap_one(t, identities, metadata, ids, nullptr, n, step, out_slots, out_evicted_slots, evicted_cap,
                     out_num_evicted, out_stats, rr, stream);
}

mpzch_status_t mpzch_remap_noalloc(const mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                                   const int64_t *ids, int64_t n, int32_t step,
                                   int64_t *out_slots,
                                   int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                                   int64_t *out_stats, void *stream)
{
    if (!t || !identities || !metadata || !out_num_evicted) return MPZCH_ERR_INVALID_ARG;
    if (n < 0 || step < 0 || evicted_cap < 0) return MPZCH_ERR_INVALID_ARG;
    if (n > MPZCH_NOALLOC_MAX_BATCH) return MPZCH_ERR_TOO_LARGE;
    if (!layout_ok(t->cfg, identities, metadata)) return MPZCH_ERR_INVALID_ARG;
    if (n > 0 && (!ids || !out_slots)) return MPZCH_ERR_INVALID_ARG;
    if (evicted_cap > 0 && !out_evicted_slots) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (n == 0) {
        TRY(fill64(out_num_evicted, 1, 0, s));
        if (out_stats) TRY(fill64(out_stats, MPZCH_STAT_COUNT, 0, s));
        return MPZCH_OK;
    }
    Scratch *sc = nullptr;
    TRY(static_scratch(s, &sc));
    Params p;
    std::memset(&p, 0, sizeof p);
    p.ids = ids;
    p.n = n;
    p.step = step;
    p.num_tables = 1;
    p.out_slots = out_slots;
    p.t0 = make_desc(t->cfg, identities, metadata, 0, evicted_cap);
    p.out_evicted = out_evicted_slots;
    p.out_num_evicted = out_num_evicted;
    p.out_stats = out_stats;
    Timing off;                                  // never enabled: records nothing, creates no event
    return run_remap(*sc, off, p, p.t0.P, p.t0.evict == 2 ? p.t0.P : 0, s);
}

mpzch_status_t mpzch_lookup(const mpzch_table_t *t, const int64_t *identities,
                            const int64_t *ids, int64_t n,
                            int64_t *out_slots, uint8_t *out_found, void *stream)
{
    if (!t || !identities_ok(t->cfg, identities)) return MPZCH_ERR_INVALID_ARG;
    if (n < 0 || n > MPZCH_MAX_BATCH) return MPZCH_ERR_INVALID_ARG;
    if (n == 0) return MPZCH_OK;
    if (!ids || !out_slots) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    int num_cus = 0;
    TRY(device_cus(&num_cus));
    Params p;
    std::memset(&p, 0, sizeof p);
    p.ids = ids;
    p.n = n;
    p.num_tables = 1;
    p.out_slots = out_slots;
    p.out_found = out_found;
    p.t0 = make_desc(t->cfg, const_cast<int64_t *>(identities), nullptr, 0, 0);
    const int grid = grid_for(n, kBlock, num_cus, discover_blocks_per_cu());
    p.num_segs = grid * kWavesPerBlock;
    p.seg_chunks = (int32_t)(((n + kWave - 1) / kWave + p.num_segs - 1) / p.num_segs);
    TIMED(t->tm, KLookup, s, (launch_discover<false>(p, grid, s)));
    return MPZCH_OK;
}

mpzch_status_t mpzch_lookup_stats(mpzch_table_t *t, const int64_t *identities,
                                  const int64_t *ids, int64_t n,
                                  int64_t *out_slots, uint8_t *out_found, int64_t *out_stats, void *stream)
{
    if (!t || !identities_ok(t->cfg, identities) || !out_stats) return MPZCH_ERR_INVALID_ARG;
    if (n < 0 || n > MPZCH_MAX_BATCH) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (n == 0) return fill64(out_stats, MPZCH_STAT_COUNT, 0, s);
    if (!ids || !out_slots) return MPZCH_ERR_INVALID_ARG;
    TRY(t->sc.query_device());
    Params p;
    std::memset(&p, 0, sizeof p);
    TRY(t->sc.ensure_ctl(&p.ctl));
    p.ids = ids;
    p.n = n;
    p.num_tables = 1;
    p.out_slots = out_slots;
    p.out_found = out_found;
    p.out_stats = out_stats;
    p.t0 = make_desc(t->cfg, const_cast<int64_t *>(identities), nullptr, 0, 0);
    const int grid = grid_for(n, kBlock, t->sc.num_cus, discover_blocks_per_cu());
    p.num_segs = grid * kWavesPerBlock;
    p.seg_chunks = (int32_t)(((n + kWave - 1) / kWave + p.num_segs - 1) / p.num_segs);
    if (!t->tm.begin(KLookup, s)) return MPZCH_ERR_HIP;
    hipLaunchKernelGGL(k_lookup_counting, dim3(grid), dim3(kBlock), 0, s, p);
    LAUNCH_CHECK();
    if (!t->tm.end(s)) return MPZCH_ERR_HIP;
    return MPZCH_OK;
}

mpzch_status_t mpzch_reset_rows(const int64_t *slots, const int64_t *num_slots_dev, int64_t slots_cap,
                                void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                const void *init_row, void *stream)
{
    if (!num_slots_dev || slots_cap < 0 || !rows || num_rows < 1) return MPZCH_ERR_INVALID_ARG;
    if (row_bytes < 4 || row_stride_bytes < row_bytes || (row_bytes & 3) || (row_stride_bytes & 3))
        return MPZCH_ERR_INVALID_ARG;
    if (((uintptr_t)rows & 3) || ((uintptr_t)init_row & 3)) return MPZCH_ERR_INVALID_ARG;
    if (slots_cap == 0) return MPZCH_OK;
    if (!slots) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const bool wide = !(row_bytes & 15) && !(row_stride_bytes & 15) && !((uintptr_t)rows & 15) &&
                      !((uintptr_t)init_row & 15);
    const int64_t chunks = wide ? row_bytes / 16 : row_bytes / 4;
    if (chunks > 0x7FFFFFFF) return MPZCH_ERR_INVALID_ARG;
    // the count lives on the device: size the grid for the capacity, bounded; the kernel strides
    int64_t want = (slots_cap * chunks + kBlock - 1) / kBlock;
    if (want > 8192) want = 8192;
    if (want < 1) want = 1;
    if (wide)
        hipLaunchKernelGGL((k_reset_rows<u32x4>), dim3((int)want), dim3(kBlock), 0, s, slots, num_slots_dev, slots_cap,
                           (char *)rows, num_rows, (int32_t)chunks, row_stride_bytes, (const u32x4 *)init_row);
    else
        hipLaunchKernelGGL((k_reset_rows<uint32_t>), dim3((int)want), dim3(kBlock), 0, s, slots, num_slots_dev,
                           slots_cap, (char *)rows, num_rows, (int32_t)chunks, row_stride_bytes,
                           (const uint32_t *)init_row);
    LAUNCH_CHECK();
    return MPZCH_OK;
}


mpzch_status_t mpzch_reset_rows_multi(const int64_t *slots, const int64_t *num_slots_dev, int64_t slots_cap,
                                      const mpzch_rows_t *tensors, int32_t num_tensors, void *stream)
{
    if (!num_slots_dev || slots_cap < 0 || !tensors || num_tensors < 1 || num_tensors > kMaxResetTensors)
        return MPZCH_ERR_INVALID_ARG;
    RowsDescs ds;
    std::memset(&ds, 0, sizeof ds);
    bool wide = true;
    for (int i = 0; i < num_tensors; ++i) {
        const mpzch_rows_t &t = tensors[i];
        if (!t.rows || t.num_rows < 1) return MPZCH_ERR_INVALID_ARG;
        const RowGeom g = row_geom(t.rows, t.row_bytes, t.row_stride_bytes, t.init_row);
        if (!g.ok) return MPZCH_ERR_INVALID_ARG;
        wide = wide && g.wide;
    }
    int64_t total = 0;
    for (int i = 0; i < num_tensors; ++i) {
        const mpzch_rows_t &t = tensors[i];
        ds.t[i].rows = (char *)t.rows;
        ds.t[i].init_row = t.init_row;
        ds.t[i].num_rows = t.num_rows;
        ds.t[i].row_stride_bytes = t.row_stride_bytes;
        ds.t[i].chunks = (int32_t)(wide ? t.row_bytes / 16 : t.row_bytes / 4);
        total += ds.t[i].chunks;
    }
    if (total > 0x7FFFFFFF) return MPZCH_ERR_INVALID_ARG;
    ds.count = num_tensors;
    ds.total_chunks = (int32_t)total;
    if (slots_cap == 0) return MPZCH_OK;
    if (!slots) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int grid = row_grid(slots_cap * total);
    if (wide) hipLaunchKernelGGL((k_reset_rows_multi<u32x4>), dim3(grid), dim3(kBlock), 0, s, slots, num_slots_dev, slots_cap, ds);
    else hipLaunchKernelGGL((k_reset_rows_multi<uint32_t>), dim3(grid), dim3(kBlock), 0, s, slots, num_slots_dev, slots_cap, ds);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

mpzch_status_t mpzch_gather_rows(const int64_t *slots, const int64_t *count_dev, int64_t cap,
                                 const void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                 void *out_rows, void *stream)
{
    if (cap < 0 || !rows || num_rows < 1 || !out_rows) return MPZCH_ERR_INVALID_ARG;
    const RowGeom g = row_geom(rows, row_bytes, row_stride_bytes, out_rows);
    if (!g.ok) return MPZCH_ERR_INVALID_ARG;
    if (cap == 0) return MPZCH_OK;
    if (!slots) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int grid = row_grid(cap * g.chunks);
    if (g.wide)
        hipLaunchKernelGGL((k_gather_rows<u32x4>), dim3(grid), dim3(kBlock), 0, s, slots, count_dev, cap, (const char *)rows,
                           num_rows, (int32_t)g.chunks, row_stride_bytes, (u32x4 *)out_rows);
    else
        hipLaunchKernelGGL((k_gather_rows<uint32_t>), dim3(grid), dim3(kBlock), 0, s, slots, count_dev, cap,
                           (const char *)rows, num_rows, (int32_t)g.chunks, row_stride_bytes, (uint32_t *)out_rows);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

mpzch_status_t mpzch_lookup_gather(const mpzch_table_t *t, const int64_t *identities,
                                   const int64_t *ids, int64_t n,
                                   const void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                   void *out_rows, int64_t *out_slots, uint8_t *out_found, void *stream)
{
    if (!t || !identities_ok(t->cfg, identities)) return MPZCH_ERR_INVALID_ARG;
    if (n < 0 || n > MPZCH_MAX_BATCH) return MPZCH_ERR_INVALID_ARG;
    if (!rows || num_rows < 1 || !out_rows) return MPZCH_ERR_INVALID_ARG;
    const RowGeom g = row_geom(rows, row_bytes, row_stride_bytes, out_rows);
    if (!g.ok || g.chunks > (1 << 20)) return MPZCH_ERR_INVALID_ARG;
    if (n == 0) return MPZCH_OK;
    if (!ids) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    int num_cus = 0;
    TRY(device_cus(&num_cus));
    Params p;
    std::memset(&p, 0, sizeof p);
    p.ids = ids;
    p.n = n;
    p.num_tables = 1;
    p.out_slots = out_slots;
    p.out_found = out_found;
    p.t0 = make_desc(t->cfg, const_cast<int64_t *>(identities), nullptr, 0, 0);
    p.g_rows = (const char *)rows;
    p.g_out = (char *)out_rows;
    p.g_num_rows = num_rows;
    p.g_stride = row_stride_bytes;
    p.g_chunks = (int32_t)g.chunks;
    p.g_wide = g.wide ? 1 : 0;
    p.g_shift = -1;
    for (int b = 0; b <= 20; ++b)
        if (g.chunks == ((int64_t)1 << b)) p.g_shift = b;
    const int grid = grid_for(n, kBlock, num_cus, discover_blocks_per_cu());
    p.num_segs = grid * kWavesPerBlock;
    p.seg_chunks = (int32_t)(((n + kWave - 1) / kWave + p.num_segs - 1) / p.num_segs);
    if (!t->tm.begin(KLookup, s)) return MPZCH_ERR_HIP;
    hipLaunchKernelGGL(k_lookup_gather, dim3(grid), dim3(kBlock), 0, s, p);
    LAUNCH_CHECK();
    if (!t->tm.end(s)) return MPZCH_ERR_HIP;
    return MPZCH_OK;
}

mpzch_status_t mpzch_collect_delta(const mpzch_table_t *t, const int64_t *identities, const int32_t *metadata,
                                   int32_t since_step, int64_t *out_slots, int64_t *out_ids, int64_t cap,
                                   int64_t *out_count, void *stream)
{
    if (!t || !identities || !metadata || !out_count || cap < 0) return MPZCH_ERR_INVALID_ARG;
    if (cap > 0 && (!out_slots || !out_ids)) return MPZCH_ERR_INVALID_ARG;
    if (!layout_ok(t->cfg, identities, metadata)) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    int num_cus = 0;
    TRY(device_cus(&num_cus));
    TRY(fill64(out_count, 1, 0, s));
    const int grid = grid_for(t->cfg.num_slots, 4 * kBlock, num_cus, 8);
    hipLaunchKernelGGL(k_collect_delta, dim3(grid), dim3(kBlock), 0, s, identities, metadata,
                       t->cfg.layout == MPZCH_LAYOUT_RECORDS ? 1 : 0, t->cfg.num_slots,
                       since_step, out_slots, out_ids, cap, (unsigned long long *)out_count);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

mpzch_status_t mpzch_apply_delta(int64_t *identities, int64_t num_slots,
                                 const int64_t *slots, const int64_t *ids, const int64_t *count_dev, int64_t cap,
                                 void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                 const void *delta_rows, void *stream)
{
    if (!identities || num_slots < 1 || cap < 0) return MPZCH_ERR_INVALID_ARG;
    RowGeom g{true, false, 1};
    if (rows) {
        if (num_rows < 1 || !delta_rows) return MPZCH_ERR_INVALID_ARG;
        g = row_geom(rows, row_bytes, row_stride_bytes, delta_rows);
        if (!g.ok) return MPZCH_ERR_INVALID_ARG;
    }
    if (cap == 0) return MPZCH_OK;
    if (!slots || !ids) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (rows) {
        const int grid = row_grid(cap * g.chunks);
        if (g.wide)
            hipLaunchKernelGGL((k_apply_delta_rows<u32x4>), dim3(grid), dim3(kBlock), 0, s, num_slots, slots, count_dev, cap,
                               (char *)rows, num_rows, (int32_t)g.chunks, row_stride_bytes, (const u32x4 *)delta_rows);
        else
            hipLaunchKernelGGL((k_apply_delta_rows<uint32_t>), dim3(grid), dim3(kBlock), 0, s, num_slots, slots, count_dev,
                               cap, (char *)rows, num_rows, (int32_t)g.chunks, row_stride_bytes,
                               (const uint32_t *)delta_rows);
        LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_apply_delta_ids, dim3(row_grid(cap)), dim3(kBlock), 0, s, identities, num_slots, slots, ids,
                       count_dev, cap);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

mpzch_status_t mpzch_group_create(mpzch_table_t *const *tables, int32_t num_tables, mpzch_group_t **out)
{
    if (!out) return MPZCH_ERR_INVALID_ARG;
    *out = nullptr;
    if (!tables || num_tables < 1 || num_tables > MPZCH_MAX_GROUP_TABLES) return MPZCH_ERR_INVALID_ARG;
    for (int i = 0; i < num_tables; ++i) {
        if (!tables[i]) return MPZCH_ERR_INVALID_ARG;
    }
    mpzch_group *g = new (std::nothrow) mpzch_group();
    if (!g) return MPZCH_ERR_ALLOC;
    for (int i = 0; i < num_tables; ++i) g->cfgs.push_back(tables[i]->cfg);
    *out = g;
    return MPZCH_OK;
}

mpzch_status_t mpzch_group_destroy(mpzch_group_t *g)
{
    if (!g) return MPZCH_OK;
    g->sc.release();
    g->tm.destroy();
    g->train.release();
    g->infer.release();
    g->rows.release();
    delete g;
    return MPZCH_OK;
}

mpzch_status_t mpzch_group_reserve(mpzch_group_t *g, int64_t max_total_values)
{
    if (!g || max_total_values < 0 || max_total_values > MPZCH_MAX_BATCH) return MPZCH_ERR_INVALID_ARG;
    return g->sc.ensure(max_total_values);
}

mpzch_status_t mpzch_remap_jagged_feature_ttl(mpzch_group_t *g, int64_t *const *identities, int32_t *const *metadata,
                                              const int64_t *values, const int32_t *ttls,
                                              const int64_t *feature_offsets,
                                              int64_t total_values, int32_t step,
                                              int64_t *out_slots,
                                              int64_t *out_evicted_slots, const int64_t *evicted_offsets,
                                              int64_t *out_num_evicted, int64_t *out_stats, void *stream)
{
    if (!g || !identities || !metadata || !feature_offsets || !evicted_offsets || !out_num_evicted)
        return MPZCH_ERR_INVALID_ARG;
    if (total_values < 0 || total_values > MPZCH_MAX_BATCH || step < 0) return MPZCH_ERR_INVALID_ARG;
    if (total_values > 0 && (!values || !out_slots)) return MPZCH_ERR_INVALID_ARG;
    const int T = (int)g->cfgs.size();
    if (ttls) {
        bool any = false;
        for (int f = 0; f < T; ++f) any = any || g->cfgs[f].kind == MPZCH_EVICT_TTL_EXPIRY;
        if (!any) return MPZCH_ERR_INVALID_ARG;          // no table of the group uses retention times
    }
    int32_t max_p = 1, max_p_lru = 0;
    std::vector<TableDesc> descs((size_t)T);
    for (int f = 0; f < T; ++f) {
        if (!identities[f] || !metadata[f]) return MPZCH_ERR_INVALID_ARG;
        if (!layout_ok(g->cfgs[f], identities[f], metadata[f])) return MPZCH_ERR_INVALID_ARG;
        const int64_t cap = evicted_offsets[f + 1] - evicted_offsets[f];
        if (cap < 0 || evicted_offsets[f] < 0) return MPZCH_ERR_INVALID_ARG;
        if (cap > 0 && !out_evicted_slots) return MPZCH_ERR_INVALID_ARG;
        descs[f] = make_desc(g->cfgs[f], identities[f], metadata[f], evicted_offsets[f], cap);
        if (descs[f].P > max_p) max_p = descs[f].P;
        if (descs[f].evict == 2 && descs[f].P > max_p_lru) max_p_lru = descs[f].P;
    }
    hipStream_t s = (hipStream_t)stream;
    if (total_values == 0) {
        TRY(fill64(out_num_evicted, T, 0, s));
        if (out_stats) TRY(fill64(out_stats, (int64_t)T * MPZCH_STAT_COUNT, 0, s));
        return MPZCH_OK;
    }
    TRY(g->sc.ensure(total_values));
    TRY(g->train.put(descs, s));
    Params p;
    std::memset(&p, 0, sizeof p);
    p.ids = values;
    p.ttls = ttls;
    p.n = total_values;
    p.step = step;
    p.num_tables = T;
    p.out_slots = out_slots;
    p.descs = g->train.dev;
    p.offsets = feature_offsets;
    p.t0 = descs[0];
    p.out_evicted = out_evicted_slots;
    p.out_num_evicted = out_num_evicted;
    p.out_stats = out_stats;
    // a group of one table still goes through the descriptor path
    if (T == 1) p.num_tables = 1;
    return run_remap(g->sc, g->tm, p, max_p, max_p_lru, s);
}

mpzch_status_t mpzch_remap_jagged(mpzch_group_t *g, int64_t *const *identities, int32_t *const *metadata,
                                  const int64_t *values, const int64_t *feature_offsets,
                                  int64_t total_values, int32_t step,
                                  int64_t *out_slots,
                                  int64_t *out_evicted_slots, const int64_t *evicted_offsets,
                                  int64_t *out_num_evicted, int64_t *out_stats, void *stream)
{
    return mpzch_remap_jagged_feature_ttl(g, identities, metadata, values, nullptr, feature_offsets, total_values, step,
                                          out_slots, out_evicted_slots, evicted_offsets, out_num_evicted, out_stats,
                                          stream);
}

mpzch_status_t mpzch_lookup_jagged(mpzch_group_t *g, const int64_t *const *identities,
                                   const int64_t *values, const int64_t *feature_offsets, int64_t total_values,
                                   int64_t *out_slots, uint8_t *out_found, void *stream)
{
    if (!g || !identities || !feature_offsets) return MPZCH_ERR_INVALID_ARG;
    if (total_values < 0 || total_values > MPZCH_MAX_BATCH) return MPZCH_ERR_INVALID_ARG;
    const int T = (int)g->cfgs.size();
    std::vector<TableDesc> descs((size_t)T);
    for (int f = 0; f < T; ++f) {
        if (!identities_ok(g->cfgs[f], identities[f])) return MPZCH_ERR_INVALID_ARG;
        descs[f] = make_desc(g->cfgs[f], const_cast<int64_t *>(identities[f]), nullptr, 0, 0);
    }
    if (total_values == 0) return MPZCH_OK;
    if (!values || !out_slots) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    TRY(g->sc.query_device());
    TRY(g->infer.put(descs, s));
    Params p;
    std::memset(&p, 0, sizeof p);
    p.ids = values;
    p.n = total_values;
    p.num_tables = T;
    p.out_slots = out_slots;
    p.out_found = out_found;
    p.descs = g->infer.dev;
    p.offsets = feature_offsets;
    p.t0 = descs[0];
    if (T == 1) p.num_tables = 1;            // a group of one table: the single-table kernel, offsets unused
    const int grid = grid_for(total_values, kBlock, g->sc.num_cus, discover_blocks_per_cu());
    p.num_segs = grid * kWavesPerBlock;
    p.seg_chunks = (int32_t)(((total_values + kWave - 1) / kWave + p.num_segs - 1) / p.num_segs);
    TIMED(g->tm, KLookup, s, (launch_discover<false>(p, grid, s)));
    return MPZCH_OK;
}

mpzch_status_t mpzch_reset_rows_jagged(mpzch_group_t *g, const int64_t *evicted_slots, const int64_t *evicted_offsets,
                                       const int64_t *num_evicted, const mpzch_rows_t *tensors, void *stream)
{
    if (!g || !evicted_offsets || !num_evicted || !tensors) return MPZCH_ERR_INVALID_ARG;
    const int T = (int)g->cfgs.size();
    std::vector<JagRows> descs((size_t)T);
    std::memset(descs.data(), 0, sizeof(JagRows) * (size_t)T);
    bool any = false;
    for (int f = 0; f < T; ++f) {
        const int64_t cap = evicted_offsets[f + 1] - evicted_offsets[f];
        if (cap < 0 || evicted_offsets[f] < 0) return MPZCH_ERR_INVALID_ARG;
        const mpzch_rows_t &t = tensors[f];
        if (!t.rows || cap == 0) continue;                   // this table has no rows to reset
        if (t.num_rows < 1) return MPZCH_ERR_INVALID_ARG;
        const RowGeom geo = row_geom(t.rows, t.row_bytes, t.row_stride_bytes, t.init_row);
        if (!geo.ok) return MPZCH_ERR_INVALID_ARG;
        JagRows &d = descs[f];
        d.rows = (char *)t.rows;
        d.init_row = t.init_row;
        d.num_rows = t.num_rows;
        d.row_stride_bytes = t.row_stride_bytes;
        d.ev_begin = evicted_offsets[f];
        d.ev_cap = cap;
        d.chunks = (int32_t)geo.chunks;
        d.wide = geo.wide ? 1 : 0;
        any = true;
    }
    if (!any) return MPZCH_OK;
    if (!evicted_slots) return MPZCH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    TRY(g->sc.query_device());
    TRY(g->rows.put(descs, s));
    hipLaunchKernelGGL(k_reset_rows_jagged, dim3(g->sc.num_cus * 8), dim3(kBlock), 0, s, evicted_slots, num_evicted,
                       g->rows.dev, T);
    LAUNCH_CHECK();
    return MPZCH_OK;
}

mpzch_status_t mpzch_set_kernel_timing(mpzch_table_t *t, int32_t enable)
{
    if (!t) return MPZCH_ERR_INVALID_ARG;
    t->tm.set_mode(enable);
    return MPZCH_OK;
}

mpzch_status_t mpzch_kernel_times(mpzch_table_t *t, const char **names, double *ms, int64_t *launches,
                                  int32_t cap, int32_t *count)
{
    if (!t || !names || !ms || !launches || !count || cap < 0) return MPZCH_ERR_INVALID_ARG;
    return t->tm.collect(names, ms, launches, cap, count);
}

mpzch_status_t mpzch_group_set_kernel_timing(mpzch_group_t *g, int32_t enable)
{
    if (!g) return MPZCH_ERR_INVALID_ARG;
    g->tm.set_mode(enable);
    return MPZCH_OK;
}

mpzch_status_t mpzch_group_kernel_times(mpzch_group_t *g, const char **names, double *ms, int64_t *launches,
                                        int32_t cap, int32_t *count)
{
    if (!g || !names || !ms || !launches || !count || cap < 0) return MPZCH_ERR_INVALID_ARG;
    return g->tm.collect(names, ms, launches, cap, count);
}

const char *mpzch_status_string(int32_t status)
{
    switch (status) {
        case MPZCH_OK: return "ok";
        case MPZCH_ERR_INVALID_ARG: return "invalid argument";
        case MPZCH_ERR_ALLOC: return "allocation failed";
        case MPZCH_ERR_HIP: return "HIP runtime error";
        case MPZCH_ERR_UNSUPPORTED: return "unsupported";
        case MPZCH_ERR_TOO_LARGE: return "size beyond the fixed maximum of this entry point";
        default: return "unknown status";
    }
}

}  // extern "C"
