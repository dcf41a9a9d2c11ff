// Device code of the MPZCH batched remap for gfx950 (wave64).
//
// Kernel sequence of one training remap (paper Sec. 3.2 / Algorithm 1, Sec. 3.4, Sec. 3.6):
//   k_discover   Pass 1 for every position.  An 8-lane group reads the aligned block of 8 slots
//                that holds the id's home slot with one coalesced access; ids and results travel
//                between the id's lane and the lanes that load for it through LDS (probe_pass);
//                the few ids whose window continues are parked in LDS and scanned 8 slots at
//                a time.  Hits store metadata = step and the output slot.  (k_lookup is the
//                same body without writes, k_discover_tables / k_lookup_tables the bodies for
//                several tables, k_discover_records the one for a table of 16-byte records.)  Each
//                wavefront owns a contiguous range of positions (a segment) and appends the
//                positions that missed to its segment's list; at the end it enters them into a
//                scratch hash set that elects, per distinct missed id, the position of its first
//                occurrence (input de-duplication of the ids that must allocate).
//   k_allocate   the elected positions claim slots.  A claim is a 64-bit atomic min of a tag
//                (round, first position) into the identities word, so a slot always ends up
//                with the claimant of the lowest (round, position); a claimant that is
//                displaced is carried on by the displacing lane from its next round.  The
//                fixed point is the unique stable assignment, the same one a sequential
//                round-major / position-minor sweep produces.
//   k_finalize   every listed position finds the slot that carries its id's claim; the elected one
//                replaces the tag by the id, sets the metadata and reports evicted slots; ids
//                without a claim fall back to home.  The scratch set entries that were used are
//                emptied again; the workgroup that finishes last publishes the call's counters.
// k_allocate / k_finalize work with one lane per claimant on the first slots of the window and
// hand the few claimants that need more to the whole wavefront (64 slots per access).  Tables
// under the LRU policy allocate in k_allocate_lru (a group of lanes per claimant) or
// k_allocate_lru_long (probe ranges beyond 64 slots).
//
// No kernel funnels work through one hot address: an atomic on a single address costs about
// 12 ns on this GPU however many lanes it serves, so miss lists are per wavefront (no shared
// cursor), counters are accumulated per workgroup and added to one of several copies, and evicted
// slots are staged in LDS and appended with one reservation per workgroup.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mpzch {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxTables = 64;
constexpr int kStatCount = 9;
constexpr int kStage = 512;            // missed positions staged per wavefront before they are entered
constexpr int kEvBuf = 256;            // evicted slots staged per wavefront before a flush

enum Stat { kHitPos = 0, kMissPos, kDistinctMiss, kInserts, kEvictions, kCollisions, kInvalidPos, kHitProbeSum, kMissProbeSum };

struct TableDesc {
    int64_t *I;            // identities
    int32_t *M;            // metadata (last-seen step)
    int64_t N;             // slots
    uint64_t seed;
    int32_t P;             // min(max_probe, N)
    int32_t ttl;
    int32_t evict;         // 0 = off, 1 = TTL (metadata = last-seen step), 2 = LRU, 3 = TTL with metadata = expiry step
    int32_t sh;            // 0: identities and metadata are two dense tensors; 1: one tensor of 16-byte records
                           // {int64 id; int32 metadata; int32 unused}, I = &record[0].id, M = &record[0].metadata
    int64_t ev_begin;      // where this table's evicted list starts in out_evicted
    int64_t ev_cap;
};

// Counters of one call.  Every workgroup adds its partial counts once, into one of kBins copies of the
// counters chosen by its index: an atomic on ONE address costs about 12 ns whatever it adds, so a
// few thousand workgroups on one address would take longer than the kernel, spread over kBins addresses
// they vanish in it.  The workgroup of k_finalize that finishes last sums the copies, publishes the
// totals and clears the block: it is all zero between calls (so a captured launch sequence can be replayed).
constexpr int kBins = 16;
struct Control {
    unsigned long long num_evicted[kMaxTables];
    unsigned long long stats[kBins][kMaxTables][kStatCount];
    unsigned long long done;       // workgroups that have finished (k_finalize: counted in the bits from kArriveShift up)
};
// k_finalize reports in by adding kArriveOne to `done`.  With one table the same atomic also reserves the
// workgroup's part of the evicted list, whose length is kept in the low bits of `done` (num_evicted[0]
// stays unused): one round trip to one address at the end of a workgroup instead of two to two.
constexpr int kArriveShift = 40;
constexpr unsigned long long kArriveOne = 1ull << kArriveShift;
constexpr unsigned long long kEvictedMask = kArriveOne - 1ull;

struct Params {
    const int64_t *ids;
    const int32_t *ttls;           // evict == 3: retention of every position's feature, or null (= the table's ttl)
    int64_t n;
    int32_t step;
    int32_t num_tables;            // 1 => t0 is used and offsets/descs are ignored
    int64_t *out_slots;
    uint8_t *out_found;            // lookup only, may be null
    // scratch.  Segment s (one wavefront of k_discover) covers the 64-position chunks
    // [s * seg_chunks, (s + 1) * seg_chunks); its missed positions are list[s * seg_chunks * 64 + k]
    // for k < seg_cnt[s]; ent and first_of run parallel to list.
    uint32_t *list;
    uint32_t *ent;                 // entry of the position's id in the scratch set
    int64_t *homes;                // home slot of the position's id
    uint32_t *first_of;            // position of the first occurrence of the position's id
    uint8_t *hint;                 // by batch position: round at which k_allocate placed the claim of the id
                                   // elected there (written for elected positions only)
    uint32_t *seg_cnt;
    int32_t seg_chunks;
    int32_t num_segs;
    uint32_t *set_slot;            // scratch hash set of batch positions, empty = 0xFFFFFFFF
    Control *ctl;
    // several tables
    const TableDesc *descs;        // device array [num_tables]
    const int64_t *offsets;        // device array [num_tables + 1]
    TableDesc t0;
    // lookup fused with the embedding gather: out[pos, :] <- rows[slot mod num_rows, :]
    const char *g_rows;
    char *g_out;
    int64_t g_num_rows;
    int64_t g_stride;              // bytes between rows
    int32_t g_chunks;              // 16-byte (g_wide) or 4-byte pieces per row
    int32_t g_wide;
    int32_t g_shift;               // log2(g_chunks) when that is a power of two, else -1
    // training remap that also resets the rows of the slots it evicts (one table; geometry in g_num_rows,
    // g_stride, g_chunks, g_wide, g_shift): rows[slot mod num_rows, :] <- init row, or zero bits
    char *r_rows;
    const void *r_init;
    // outputs
    int64_t *out_evicted;
    int64_t *out_num_evicted;
    int64_t *out_stats;
};

// ------------------------------------------------------------------ arithmetic
__device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ int64_t home_slot(int64_t id, uint64_t seed, int64_t n_slots)
{
    return (int64_t)__umul64hi(mix64((uint64_t)id ^ seed), (uint64_t)n_slots);
}

// Claim tags live in the identities word while a call is in flight.  They are below every
// valid id and below the empty marker, and a smaller tag is a better claim.
constexpr uint64_t kTagBase = 0x8000000000000000ull;
constexpr int kTagRoundShift = 33;

__device__ __forceinline__ int64_t make_tag(uint32_t round, uint32_t pos, uint32_t was_occupied)
{
    return (int64_t)(kTagBase | ((uint64_t)round << kTagRoundShift) | ((uint64_t)pos << 1) | was_occupied);
}
__device__ __forceinline__ bool is_tag(int64_t v) { return v < -1; }
__device__ __forceinline__ uint32_t tag_pos(int64_t v) { return (uint32_t)(((uint64_t)v >> 1) & 0xFFFFFFFFull); }
__device__ __forceinline__ uint32_t tag_round(int64_t v) { return (uint32_t)(((uint64_t)v & ~kTagBase) >> kTagRoundShift); }
__device__ __forceinline__ uint32_t tag_occ(int64_t v) { return (uint32_t)((uint64_t)v & 1u); }

__device__ __forceinline__ int64_t shfl64(int64_t v, int src)
{
    int lo = __shfl((int)(uint32_t)(uint64_t)v, src);
    int hi = __shfl((int)(uint32_t)((uint64_t)v >> 32), src);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// table owning position pos (largest f with offsets[f] <= pos)
__device__ __forceinline__ int find_table(const int64_t *offsets, int num_tables, int64_t pos)
{
    int lo = 0, hi = num_tables - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (offsets[mid] <= pos) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ int64_t wrap(int64_t s, int64_t n) { return s >= n ? s - n : s; }

// Device-side view of a TableDesc.  A pointer read from a descriptor in memory has lost the
// "global" address space that kernel arguments carry, and accesses through it become flat_
// instructions, which also count against the LDS wait counter.  All table state is device memory,
// and the view's pointer types say so.
template <typename T>
using global_ptr = T __attribute__((address_space(1))) *;

struct Tab {
    global_ptr<int64_t> I;
    global_ptr<int32_t> M;
    int64_t N;
    uint64_t seed;
    int32_t P;
    int32_t ttl;
    int32_t evict;
    int32_t sh;
};

// Where slot s lives.  Two dense tensors (sh = 0): I[s], M[s].  One tensor of 16-byte records (sh = 1): the id of
// slot s is the int64 at I + 2 s, its metadata the int32 at M + 4 s -- the line that a probe fetches then also
// holds the metadata word that a hit refreshes.
__device__ __forceinline__ global_ptr<int64_t> id_at(const Tab &d, int64_t s) { return d.I + (s << d.sh); }
__device__ __forceinline__ global_ptr<int32_t> meta_at(const Tab &d, int64_t s) { return d.M + (s << (2 * d.sh)); }
// identities of slot s's aligned block of 8 (64 bytes, or 128 bytes of records): how far s lies into it
__device__ __forceinline__ int block_offset(const Tab &d, int64_t s, int slots)
{
    return (int)((s + (int64_t)(((uintptr_t)d.I >> (3 + d.sh)) & (uintptr_t)(slots - 1))) & (slots - 1));
}

__device__ __forceinline__ Tab view(const TableDesc &d)
{
    Tab t;
    t.I = (global_ptr<int64_t>)d.I;
    t.M = (global_ptr<int32_t>)d.M;
    t.N = d.N;
    t.seed = d.seed;
    t.P = d.P;
    t.ttl = d.ttl;
    t.evict = d.evict;
    t.sh = d.sh;
    return t;
}

// A value that is the same in every lane, read from lane 0 so that the compiler keeps it in scalar
// registers (a descriptor loaded from memory arrives in vector registers: the kernels also store to
// global memory, so the load cannot be a scalar one).
__device__ __forceinline__ int32_t uniform32(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uniform64(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uint64_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ Tab uniform(const Tab &d)
{
    Tab t;
    t.I = (global_ptr<int64_t>)(uintptr_t)uniform64((int64_t)(uintptr_t)(int64_t *)d.I);
    t.M = (global_ptr<int32_t>)(uintptr_t)uniform64((int64_t)(uintptr_t)(int32_t *)d.M);
    t.N = uniform64(d.N);
    t.seed = (uint64_t)uniform64((int64_t)d.seed);
    t.P = uniform32(d.P);
    t.ttl = uniform32(d.ttl);
    t.evict = uniform32(d.evict);
    t.sh = uniform32(d.sh);
    return t;
}

// Metadata written for the id at batch position pos: the step (last seen), or with per-feature TTL
// (Sec. 3.4) the step after which the id is expired: now + duration of its feature.
__device__ __forceinline__ int32_t meta_value(const Params &p, const Tab &d, int64_t pos)
{
    if (d.evict != 3) return p.step;
    return p.step + (p.ttls ? p.ttls[pos] : d.ttl);
}

// Metadata write on behalf of one batch position.  With last-seen metadata every writer of a call
// stores the same step.  With per-feature expiry times (Sec. 3.4, second paragraph) the writers of one
// slot -- the copies of the id that lives there, which may come from features of different retention,
// and the ids that fall back to it as their home -- carry different values; the slot keeps the latest
// expiry step any of them asks for: a refresh never moves it backward, so a short-lived feature
// cannot cut short the retention a long-lived one gave the slot, and the result does not depend on
// the order of the writers.  (A slot that is claimed held -1 or an expired value, which is below
// every value written at this step.)
__device__ __forceinline__ void store_meta(const Tab &d, int64_t s, int32_t value)
{
    if (d.evict == 3) __hip_atomic_fetch_max(meta_at(d, s), value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *meta_at(d, s) = value;
}

// TTL test of Sec. 3.4 on metadata m of a slot that holds an id
__device__ __forceinline__ bool is_expired(int32_t evict, int32_t ttl, int32_t step, int32_t m)
{
    if (evict == 1) return (int64_t)step - (int64_t)m > (int64_t)ttl;
    if (evict == 3) return m < step;
    return false;
}

// ------------------------------------------------------------------ scratch set
constexpr uint64_t kSetSeed = 0x2545F4914F6CDD1Dull;
constexpr uint32_t kSetEmpty = 0xFFFFFFFFu;

// The scratch set elects, per distinct missed id, the smallest batch position holding it.  An
// entry is one 32-bit word: a batch position (the id it stands for is ids[position]) or empty.
// Inserting (id, pos) into the region [base, base + size): claim the first empty entry of the
// probe sequence with one compare-and-swap, or, on meeting an entry of the same id, lower it to
// min(entry, pos).  An entry never changes the id it stands for, so concurrent inserts agree.
// size >= 2 * (number of inserts into the region), so the unbounded probe always ends.
// Returns the entry index.
__device__ __forceinline__ uint32_t set_insert(const Params &p, int64_t id, uint32_t pos, uint64_t base, uint64_t size)
{
    uint64_t e = base + __umul64hi(mix64((uint64_t)id ^ kSetSeed), size);
    const uint64_t end = base + size;
    for (;;) {
        uint32_t expected = kSetEmpty;
        if (__hip_atomic_compare_exchange_strong(&p.set_slot[e], &expected, pos, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT))
            break;                                            // first of its id so far
        if ((int64_t)expected < p.n && p.ids[expected] == id) {   // (an entry is always a position of this batch)
            if (pos < expected) __hip_atomic_fetch_min(&p.set_slot[e], pos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
        if (++e == end) e = base;
    }
    return (uint32_t)e;
}

// ------------------------------------------------------------------ small wavefront helpers
__device__ __forceinline__ unsigned long long wave_sum(unsigned long long x)
{
    // rotation sum: afterwards every lane holds the wavefront total
    const int lane = lane_id();
    for (int o = 32; o > 0; o >>= 1) x += (unsigned long long)shfl64((int64_t)x, (lane + o) & 63);
    return x;
}

// Hands the next (64 / G) set bits of amask to the G-lane groups of the wavefront: returns this
// group's bit index or -1, and removes the bits that were handed out.
template <int G>
__device__ __forceinline__ int next_bits(uint64_t &amask, int g)
{
    constexpr int GPW = kWave / G;
    int b = -1;
    uint64_t m = amask;
#pragma unroll
    for (int gg = 0; gg < GPW; ++gg) {
        const int bb = m ? __ffsll((unsigned long long)m) - 1 : -1;
        if (gg == g) b = bb;
        m &= m - 1;
    }
    amask = m;
    return b;
}

// Region of the scratch set that serves the table owning `pos`: twice the number of positions
// of that table, so it can never fill up.  The clamps keep the region inside [0, 2n) even if the
// feature offsets break their contract.
__device__ __forceinline__ void set_region(const Params &p, int64_t pos, uint64_t &base, uint64_t &size)
{
    if (p.num_tables <= 1) { base = 0; size = 2ull * (uint64_t)p.n; return; }
    const int f = find_table(p.offsets, p.num_tables, pos);
    int64_t lo = p.offsets[f], hi = p.offsets[f + 1];
    if (f == p.num_tables - 1 || hi > p.n) hi = p.n;
    if (hi <= pos) hi = pos + 1;
    if (lo > pos) lo = pos;
    if (lo < 0) lo = 0;
    base = 2ull * (uint64_t)lo;
    size = 2ull * (uint64_t)(hi - lo);
}

__device__ __forceinline__ unsigned long long *stat_word(const Params &p, int table, int k)
{
    return &p.ctl->stats[blockIdx.x % kBins][table][k];
}

// Sums per-lane counters over the workgroup and adds them to this workgroup's copy of the call's
// counters: one atomic per counter when all its wavefronts ended on the same table (the rule), one
// per wavefront and counter otherwise.  Must be reached by all threads of the workgroup.
__device__ __forceinline__ void block_stat_add(const Params &p, const int *idx, const unsigned long long *vals,
                                               int count, int table, unsigned long long (*s_red)[kStatCount],
                                               int *s_tab)
{
    const int lane = lane_id(), w = threadIdx.x / kWave;
    for (int k = 0; k < count; ++k) {
        const unsigned long long t = wave_sum(vals[k]);
        if (lane == 0) s_red[w][idx[k]] = t;
    }
    if (lane == 0) s_tab[w] = table;
    __syncthreads();
    if ((int)threadIdx.x < count) {
        const int k = idx[threadIdx.x];
        bool same = true;
        for (int i = 1; i < kWavesPerBlock; ++i) same = same && s_tab[i] == s_tab[0];
        if (same) {
            unsigned long long v = 0;
            for (int i = 0; i < kWavesPerBlock; ++i) v += s_red[i][k];
            if (v) atomicAdd(stat_word(p, s_tab[0], k), v);
        } else {
            for (int i = 0; i < kWavesPerBlock; ++i)
                if (s_red[i][k]) atomicAdd(stat_word(p, s_tab[i], k), s_red[i][k]);
        }
    }
}

// Sums the kBins copies of the call's counters, writes out_num_evicted / out_stats and clears the block.
// Run by the workgroup that finishes last (of k_finalize; of a counting lookup).
__device__ __forceinline__ void publish_counters(const Params &p, unsigned long long (*s_bins)[kStatCount])
{
    if (p.out_num_evicted) {
        if (p.num_tables > 1) {
            for (int i = threadIdx.x; i < p.num_tables; i += kBlock)
                p.out_num_evicted[i] =
                    (int64_t)__hip_atomic_load(&p.ctl->num_evicted[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else if (threadIdx.x == 0) {
            p.out_num_evicted[0] =
                (int64_t)(__hip_atomic_load(&p.ctl->done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kEvictedMask);
        }
    }
    if (p.out_stats) {
        const int nbins = p.num_tables * kStatCount;
        for (int i = threadIdx.x; i < nbins; i += kBlock) {
            unsigned long long v = 0;
            for (int b = 0; b < kBins; ++b)
                v += __hip_atomic_load(&p.ctl->stats[b][i / kStatCount][i % kStatCount], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            s_bins[i / kStatCount][i % kStatCount] = v;
        }
        __syncthreads();
        for (int t = threadIdx.x; t < p.num_tables; t += kBlock)
            s_bins[t][kDistinctMiss] = s_bins[t][kInserts] + s_bins[t][kEvictions] + s_bins[t][kCollisions];
        __syncthreads();
        for (int i = threadIdx.x; i < nbins; i += kBlock)
            p.out_stats[i] = (int64_t)s_bins[i / kStatCount][i % kStatCount];
    }
    __syncthreads();
    unsigned long long *z = reinterpret_cast<unsigned long long *>(p.ctl);
    for (int i = threadIdx.x; i < (int)(sizeof(Control) / sizeof(unsigned long long)); i += kBlock) z[i] = 0ull;
}

// ------------------------------------------------------------------ Pass 1 (discovery)
// One probe pass over the 64 ids held one per lane: the id of lane L is compared with the G
// slots of rounds [q, q + G) of its window (q may be negative: rounds below 0 do not exist;
// q >= d.P switches the lane off).  A G-lane group serves one id per access, so with q chosen
// such that home + q is a multiple of G slots every access reads one aligned block of 8 G bytes.
// All G accesses are issued before the first result is looked at; a lane without a slot to
// look at re-reads the home slot (a valid address, same or neighbouring line; slot 0 if the id
// is switched off or belongs to another table), so the loads carry no branch and stay in flight
// together.  d is wave-uniform.  Returns the round of the match; kProbeGoOn when the id is not among
// these slots; or, when in addition one of them is empty, a value <= kProbeAbsent that names the round
// of the first empty slot (probe_absent / absent_len): a slot never becomes empty again once it was
// occupied, so no resident id lies beyond an empty slot of its window and the search can end there.
constexpr int kFirstG = 8;             // slots looked at by the first pass: the aligned 64 bytes that hold the home slot
constexpr int kProbeGoOn = -1;
constexpr int kProbeAbsent = -2;

__device__ __forceinline__ int probe_absent(int empty_round) { return kProbeAbsent - empty_round; }
// slots of the window read until the search ended: up to and including the first empty one
__device__ __forceinline__ int absent_len(int code) { return -code - 1; }

// What the lane that holds an id leaves in LDS for the lanes that load for it: the id, and `where`
// = address of the identity of the first slot to read (bits 0..47: device addresses have no more)
// with, in bit 48 + r, whether round q + r exists (r < G).
struct alignas(16) ProbeReq {
    int64_t id;
    uint64_t where;
};
constexpr int kWhereAddrBits = 48;

// the loads of one pass: lane r of a group reads slot number k(r) behind the first one, where k counts the rounds
// that exist below its own -- its own slot when its round exists, else the first slot (r < r_lo) or the one after
// the last (r >= r_hi): valid addresses in or next to the line that is fetched anyway.  Slots past the end of the
// table go on at slot 0.
// NT: the loads are marked non-temporal (see k_discover_streaming).
template <int G, bool NT>
__device__ __forceinline__ void probe_loads(const Tab &d, const ProbeReq *s_req, int64_t (&v)[G])
{
    constexpr int IPI = kWave / G;
    const int lane = lane_id();
    const int g = lane / G, r = lane % G;
    const uint32_t below = (1u << r) - 1u;
    const int sh3 = 3 + d.sh;
    const uint64_t table_bytes = (uint64_t)d.N << sh3;
    const uint64_t table_end = (uint64_t)(uintptr_t)(int64_t *)d.I + table_bytes;
#pragma unroll
    for (int t = 0; t < G; ++t) {
        const uint64_t where = s_req[t * IPI + g].where;
        const uint32_t k = (uint32_t)__popc((uint32_t)(where >> kWhereAddrBits) & below);
        uint64_t a = (where & ((1ull << kWhereAddrBits) - 1ull)) + (uint64_t)(k << sh3);
        if (a >= table_end) a -= table_bytes;
        if constexpr (NT) v[t] = __builtin_nontemporal_load((global_ptr<int64_t>)(uintptr_t)a);
        else v[t] = *(global_ptr<int64_t>)(uintptr_t)a;
    }
}

// s_req: 64 requests, s_code: 64 * G bytes, both this wavefront's own areas of LDS.  The G lanes of
// a group read G consecutive slots of one id per access; what each saw (1 = the id, 2 = an empty
// slot, 0 = neither) goes back through LDS as one byte per slot, and the id's own lane reads its G
// bytes at once and drops those of rounds that do not exist: no cross-lane operation depends on a
// load, and nothing branches.
template <int G, bool NT = false>
__device__ __forceinline__ int probe_pass(const Tab &d, int64_t id, int64_t home, int q, ProbeReq *s_req,
                                          uint8_t *s_code)
{
    static_assert(G == 8, "the codes of one id are read back as one 64-bit word");
    constexpr int IPI = kWave / G;
    const int lane = lane_id();
    const int g = lane / G;
    // the rounds of [q, q + G) that exist are r_lo <= r < r_hi; none when the lane is switched off
    const int r_lo = q < 0 ? -q : 0;
    const int r_hi = d.P - q < G ? d.P - q : G;
    const int count = r_hi - r_lo;
    const bool on = count > 0;
    const uint32_t rounds = on ? ((1u << r_hi) - 1u) & ~((1u << r_lo) - 1u) : 0u;
    // the slots read for this id are first_slot .. first_slot + count (the last by lanes without a round)
    const int64_t first_slot = on ? wrap(home + (q + r_lo), d.N) : 0;
    s_req[lane] = ProbeReq{id, (uint64_t)(uintptr_t)(int64_t *)id_at(d, first_slot) | ((uint64_t)rounds << kWhereAddrBits)};
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    int64_t v[G];
    probe_loads<G, NT>(d, s_req, v);
#pragma unroll
    for (int t = 0; t < G; ++t) {
        const int64_t gid = s_req[t * IPI + g].id;
        s_code[t * kWave + lane] = v[t] == gid ? 1 : (v[t] == -1 ? 2 : 0);        // = byte r of id t * IPI + g
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // the lowest set bit of the bytes of the rounds that exist: bit 8 j = found at round q + r_lo + j,
    // bit 8 j + 1 = that round's slot is empty
    const uint64_t x = *reinterpret_cast<const uint64_t *>(s_code + lane * G) >> (8 * r_lo);
    const int bit = __ffsll((unsigned long long)x) - 1;
    const int j = bit >> 3;
    const int round = q + r_lo + j;
    const int found = (x == 0 || j >= count) ? kProbeGoOn : ((bit & 1) ? probe_absent(round) : round);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");    // the areas are written again by the next pass
    return found;
}

// out[pos, :] <- rows[slot mod num_rows, :] for the positions of the active lanes (Sec. 3.7: the lookup
// fused with the embedding gather).  The 64 rows are copied by the whole wavefront, consecutive lanes
// moving consecutive 16-byte (or 4-byte) pieces of a row, several loads in flight per lane.
template <typename VEC>
__device__ __forceinline__ void gather_rows_wave(const Params &p, uint64_t am, int64_t pos, int64_t row)
{
    constexpr int U = 4;
    const int lane = lane_id();
    const int C = p.g_chunks;
    const int total = kWave * C;
    for (int i0 = 0; i0 < total; i0 += kWave * U) {
        VEC v[U];
        int64_t dst[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = i0 + u * kWave + lane;
            const bool in = idx < total;
            const int src = in ? (p.g_shift >= 0 ? idx >> p.g_shift : idx / C) : 0;
            const int c = idx - src * C;
            const int64_t srow = shfl64(row, src);
            const int64_t spos = shfl64(pos, src);
            ok[u] = in && ((am >> src) & 1ull);
            dst[u] = spos * C + c;
            v[u] = VEC(0);
            if (ok[u]) v[u] = reinterpret_cast<const VEC *>(p.g_rows + srow * p.g_stride)[c];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) __builtin_nontemporal_store(v[u], reinterpret_cast<VEC *>(p.g_out) + dst[u]);
    }
}

__device__ __forceinline__ void gather_wave(const Params &p, bool active, int64_t pos, int64_t slot)
{
    const uint64_t am = __ballot(active);
    if (!am) return;
    int64_t row = active ? slot : 0;
    if (row >= p.g_num_rows) row %= p.g_num_rows;
    if (p.g_wide) gather_rows_wave<u32x4>(p, am, pos, row);
    else gather_rows_wave<uint32_t>(p, am, pos, row);
}

// Every wavefront owns one segment of positions.  Per 64-position chunk it probes the line that
// holds each id's home slot.  Ids that were not found there but whose window goes on are parked
// in LDS (position, next round) and resolved later, 64 at a time, so that the second
// memory round trip is paid once per 64 parked ids instead of once per chunk.  What remains
// unfound is the segment's miss list.
template <bool TRAIN, bool MULTI, bool GATHER, bool COUNT = TRAIN, bool NT = false>
__device__ __forceinline__ void discover_body(const Params &p)
{
    __shared__ uint32_t s_pos[kWavesPerBlock][kStage];
    __shared__ int32_t s_q[kWavesPerBlock][kStage];      // > 0: next round to look at; < 0: absent, -(slots read)
    __shared__ unsigned long long s_red[kWavesPerBlock][kStatCount];
    __shared__ int s_tab[kWavesPerBlock];
    __shared__ ProbeReq s_req[kWavesPerBlock][kWave];
    __shared__ __attribute__((aligned(16))) uint8_t s_code[kWavesPerBlock][kWave * kFirstG];
    constexpr int kNextG = 8;                    // slots per id and access of the passes after the first

    const int lane = lane_id();
    const int w = threadIdx.x / kWave;
    const int64_t seg = (int64_t)blockIdx.x * kWavesPerBlock + w;       // this wavefront's segment
    const int64_t num_chunks = (p.n + kWave - 1) / kWave;
    const int64_t c_begin = seg * p.seg_chunks;
    const int64_t c_end = c_begin + p.seg_chunks < num_chunks ? c_begin + p.seg_chunks : num_chunks;
    const int64_t seg_base = c_begin * kWave;
    constexpr bool multi = MULTI;
    const bool want_stats = COUNT && p.out_stats != nullptr;

    // per-lane counters of the table currently being processed
    unsigned long long st_hit = 0, st_miss = 0, st_inv = 0, st_probe = 0, st_mlen = 0;
    int st_table = 0;
    int staged = 0, flushed = 0;                 // wave-uniform: parked ids in LDS / misses already listed

    // Several tables: the table that owns the positions this wavefront is working through, with the
    // range of positions it owns (all wave-uniform).  Positions arrive in ascending order, so the
    // search through the offsets and the load of the descriptor -- a chain of dependent loads in
    // front of every hash -- are paid when the range is left, not once per chunk.
    int t_f = 0;
    int64_t t_lo = 0, t_hi = 0;
    Tab t_d = view(p.t0);
    auto table_at = [&](int64_t upos) {
        if (upos >= t_lo && upos < t_hi) return;
        t_f = __builtin_amdgcn_readfirstlane(find_table(p.offsets, p.num_tables, upos));
        // find_table skips empty features that share this offset; the clamps keep every loop
        // finite and every range inside the batch even if the offsets break their contract
        int64_t lo = p.offsets[t_f], hi = p.offsets[t_f + 1];
        if (t_f == p.num_tables - 1 || hi > p.n) hi = p.n;
        if (hi <= upos) hi = upos + 1;
        if (lo > upos) lo = upos;
        if (lo < 0) lo = 0;
        t_lo = uniform64(lo);
        t_hi = uniform64(hi);
        t_d = uniform(view(p.descs[t_f]));
    };

    // counters are kept for one table at a time
    auto stats_table = [&](int f) {
        if (!want_stats || f == st_table) return;
        // table changed inside this wavefront's range (rare): hand the counters over
        const unsigned long long a = wave_sum(st_hit), b = wave_sum(st_miss), x = wave_sum(st_inv), y = wave_sum(st_probe),
                                 z = wave_sum(st_mlen);
        if (lane == 0) {
            if (a) atomicAdd(stat_word(p, st_table, kHitPos), a);
            if (b) atomicAdd(stat_word(p, st_table, kMissPos), b);
            if (x) atomicAdd(stat_word(p, st_table, kInvalidPos), x);
            if (y) atomicAdd(stat_word(p, st_table, kHitProbeSum), y);
            if (z) atomicAdd(stat_word(p, st_table, kMissProbeSum), z);
        }
        st_hit = st_miss = st_inv = st_probe = st_mlen = 0;
        st_table = f;
    };
    // a position whose id is resident at `dist` probes from home
    // (the first pass stores the outputs of its whole chunk itself: emit = false)
    auto finish_hit = [&](const Tab &d, int64_t pos, int64_t home, int dist, bool emit) {
        const int64_t slot = wrap(home + dist, d.N);
        if (TRAIN) {
            store_meta(d, slot, meta_value(p, d, pos));   // "Update": refresh the resident's metadata
        }
        if (COUNT) {
            st_hit++;
            st_probe += (unsigned long long)(dist + 1);
        }
        if (emit) {
            if (!GATHER || p.out_slots) p.out_slots[pos] = slot;
            if (!TRAIN && p.out_found) p.out_found[pos] = 1;
        }
    };

    // probes the parked ids until found or their window ends; enters the rest into the scratch set
    auto resolve_stage = [&]() {
        // the outputs stored by the first pass are performed before any lane rewrites them below
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        int nmiss = 0;
        bool all_cached = true;                 // wave-uniform: every parked position is of the cached table
        for (int e0 = 0; e0 < staged; e0 += kWave) {
            const bool have = e0 + lane < staged;
            const uint32_t pos = have ? s_pos[w][e0 + lane] : 0;
            const int q0 = have ? s_q[w][e0 + lane] : 0;
            const int64_t id = have ? p.ids[pos] : -1;
            // parked positions nearly always belong to the table of the chunks just read
            const bool cached = !multi || __all(!have || ((int64_t)pos >= t_lo && (int64_t)pos < t_hi));
            if (!cached) all_cached = false;
            const int f = (have && !cached) ? find_table(p.offsets, p.num_tables, (int64_t)pos) : t_f;
            bool todo = have;
            while (__any(todo)) {
                const int f0 = cached ? t_f : __shfl(f, __ffsll((unsigned long long)__ballot(todo)) - 1);
                const bool mine = todo && f == f0;
                Tab d = t_d;                                    // one table: t_d is the table
                if (multi && !cached) d = uniform(view(p.descs[f0]));
                stats_table(f0);
                const int64_t home = mine ? home_slot(id, d.seed, d.N) : 0;
                int dist = -1;
                int mlen = q0 < 0 ? -q0 : 0;                // > 0: the search has ended at an empty slot
                int q = q0 > 0 ? q0 : d.P;
                for (;;) {
                    const bool need = mine && dist < 0 && mlen == 0 && q < d.P;
                    if (!__any(need)) break;
                    const int got = probe_pass<kNextG, NT>(d, id, home, need ? q : d.P, s_req[w], s_code[w]);
                    if (need) {
                        if (got >= 0) dist = got;
                        else if (got <= kProbeAbsent) mlen = absent_len(got);   // an empty slot ends the search
                        else q += kNextG;
                    }
                }
                if (mine && dist >= 0) finish_hit(d, (int64_t)pos, home, dist, true);
                const bool miss = mine && dist < 0;
                const uint64_t mb = __ballot(miss);
                if (miss && TRAIN) {
                    const int at = nmiss + __popcll(mb & ((1ull << lane) - 1ull));      // slots already consumed
                    s_pos[w][at] = pos;
                }
                if (miss && COUNT) {
                    st_miss++;
                    st_mlen += (unsigned long long)(mlen ? mlen : d.P);
                }
                // lookup: the first pass has already stored home and "not found"
                if (GATHER) gather_wave(p, mine, (int64_t)pos, dist >= 0 ? wrap(home + dist, d.N) : home);
                nmiss += __popcll(mb);
                todo = todo && !mine;
            }
        }
        if (TRAIN) {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            // (read through lane 0: as plain copies the compiler would fold them with the per-lane descriptor
            // loads of the last branch below into loads through a selected pointer, which puts t_d in memory)
            const uint64_t c_seed = (uint64_t)uniform64((int64_t)t_d.seed);
            const int64_t c_n = uniform64(t_d.N);
            for (int j = lane; j < nmiss; j += kWave) {
                const uint32_t pos = s_pos[w][j];
                const int64_t id = p.ids[pos];
                uint64_t sb, ss;
                int64_t home;
                if (!multi) {
                    sb = 0;
                    ss = 2ull * (uint64_t)p.n;
                    home = home_slot(id, p.t0.seed, p.t0.N);
                } else if (all_cached) {
                    sb = 2ull * (uint64_t)t_lo;
                    ss = 2ull * (uint64_t)(t_hi - t_lo);
                    home = home_slot(id, c_seed, c_n);
                } else {
                    set_region(p, (int64_t)pos, sb, ss);
                    const TableDesc &td = p.descs[find_table(p.offsets, p.num_tables, (int64_t)pos)];
                    home = home_slot(id, td.seed, td.N);
                }
                const uint32_t e = set_insert(p, id, pos, sb, ss);
                p.list[seg_base + flushed + j] = pos;
                p.ent[seg_base + flushed + j] = e;
                p.homes[seg_base + flushed + j] = home;
            }
            flushed += nmiss;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        staged = 0;
    };

    // the ids of the next chunk are requested while the current one is probed
    int64_t id_next = (c_begin < c_end && c_begin * kWave + lane < p.n) ? p.ids[c_begin * kWave + lane] : -1;
    for (int64_t c = c_begin; c < c_end; ++c) {
        const int64_t base = c * kWave;
        const int64_t pos = base + lane;
        const bool in_range = pos < p.n;
        const int64_t id = id_next;
        id_next = (c + 1 < c_end && pos + kWave < p.n) ? p.ids[pos + kWave] : -1;
        bool todo = in_range;
        // every pass handles the lanes that belong to one table (one pass unless the chunk
        // straddles a feature boundary)
        while (__any(todo)) {
            Tab d;
            int f = 0;
            bool mine = todo;
            if (multi) {
                const uint64_t tb = __ballot(todo);
                table_at(base + __ffsll((unsigned long long)tb) - 1);
                f = t_f;
                d = t_d;
                mine = todo && pos < t_hi;
            } else {
                d = view(p.t0);
            }
            stats_table(f);

            const bool valid = mine && id >= 0;
            const int64_t home = mine ? home_slot(id, d.seed, d.N) : 0;
            // first pass: the aligned 64 bytes that hold the home slot
            const int o = block_offset(d, home, kFirstG);
            int res = probe_pass<kFirstG, NT>(d, id, home, valid ? -o : d.P, s_req[w], s_code[w]);
            if (res == kProbeGoOn && kFirstG - o >= d.P) res = probe_absent(d.P - 1);    // the whole window was read
            const bool hit = valid && res >= 0;
            if (hit) finish_hit(d, pos, home, res, false);
            else if (COUNT && mine && !valid) st_inv++;
            if (COUNT && !TRAIN && valid && res <= kProbeAbsent) {           // a lookup miss decided here is final
                st_miss++;
                st_mlen += (unsigned long long)absent_len(res);
            }
            // One store for the whole chunk keeps the 64-byte sectors of the outputs complete (a
            // sector written with holes leaves the cache as narrow writes).  A position that is
            // not decided yet gets its home slot: final for a negative id (home of its bit
            // pattern) and for a lookup miss, rewritten later otherwise.
            const int64_t slot = hit ? wrap(home + res, d.N) : home;
            if (mine) {
                // (non-temporal: the outputs are not read by this call; nine in ten are final here)
                if (!GATHER || p.out_slots) __builtin_nontemporal_store(slot, &p.out_slots[pos]);
                if (!TRAIN && p.out_found) p.out_found[pos] = hit ? 1 : 0;
            }
            // not found so far: parked when its window goes on, or (training) to be listed as a miss
            const bool park = valid && (res == kProbeGoOn || (TRAIN && res <= kProbeAbsent));
            const uint64_t pb = __ballot(park);
            if (park) {
                const int at = staged + __popcll(pb & ((1ull << lane) - 1ull));
                s_pos[w][at] = (uint32_t)pos;
                s_q[w][at] = res <= kProbeAbsent ? -absent_len(res) : kFirstG - o;
            }
            staged += __popcll(pb);
            if (GATHER) gather_wave(p, mine && !park, pos, slot);
            todo = todo && !mine;
        }
        if (staged > kStage - kWave) resolve_stage();
    }
    resolve_stage();
    if (TRAIN && lane == 0 && seg < p.num_segs) p.seg_cnt[seg] = (uint32_t)flushed;
    if (want_stats) {
        const int idx[5] = {kHitPos, kMissPos, kInvalidPos, kHitProbeSum, kMissProbeSum};
        const unsigned long long vals[5] = {st_hit, st_miss, st_inv, st_probe, st_mlen};
        block_stat_add(p, idx, vals, 5, st_table, s_red, s_tab);
    }
    if constexpr (COUNT && !TRAIN) {
        // a counting lookup publishes its own counters (see finalize_body for the training remap)
        __shared__ unsigned long long s_bins[kMaxTables][kStatCount];
        __shared__ bool s_last;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0) s_last = atomicAdd(&p.ctl->done, 1ull) == (unsigned long long)(gridDim.x - 1);
        __syncthreads();
        if (s_last) publish_counters(p, s_bins);
    }
}

// The kernels around the one body.  At most four wavefronts per SIMD (the compiler then has 128 registers
// and needs about 90): the pass is bound by memory, and measured within 2 % of its best from three to six
// wavefronts for both table layouts; fewer hide the latency of the loads less well, more only add to the
// queues of the memory system.
__global__ __launch_bounds__(kBlock, 4) void k_discover(Params p)
{
    discover_body<true, false, false>(p);
}

// The same pass with the identities read by non-temporal loads, for a two-tensor table far larger than the
// caches: a line of identities is not used again before it is evicted anyway, and not keeping it leaves the L2
// to the lines of metadata that the hits write into (headline with two tensors: 0.295 -> 0.253 ms).  Not for
// records -- there the refresh goes into the very line the probe has fetched (0.218 -> 0.277 ms with such
// loads) -- and not for lookups, whose repeated ids do hit in the L2 (config 3: 0.029 -> 0.034 ms).
__global__ __launch_bounds__(kBlock, 4) void k_discover_streaming(Params p)
{
    discover_body<true, false, false, true, true>(p);
}

// the same pass over a table kept as 16-byte records: the metadata store lands in the line just read
__global__ __launch_bounds__(kBlock, 4) void k_discover_records(Params p)
{
    discover_body<true, false, false>(p);
}

__global__ __launch_bounds__(kBlock, 4) void k_lookup(Params p)
{
    discover_body<false, false, false>(p);
}

__global__ __launch_bounds__(kBlock, 2) void k_lookup_gather(Params p)
{
    discover_body<false, false, true>(p);
}

__global__ __launch_bounds__(kBlock, 3) void k_lookup_counting(Params p)
{
    discover_body<false, false, false, true>(p);
}

__global__ __launch_bounds__(kBlock, 4) void k_discover_tables(Params p)
{
    discover_body<true, true, false>(p);
}

__global__ __launch_bounds__(kBlock, 4) void k_lookup_tables(Params p)
{
    discover_body<false, true, false>(p);
}

// Several tables: the table of a whole segment of positions [seg_base, seg_base + seg_len), when one
// table owns them all (the rule: a segment is a few thousand positions, a feature's share of the
// batch many times that).  Its number and descriptor are then wave-uniform and read once per segment
// instead of once per lane and list entry.  Returns false when the segment straddles a boundary.
__device__ __forceinline__ bool segment_table(const Params &p, int64_t seg_base, int64_t seg_len, int &f, Tab &d)
{
    f = __builtin_amdgcn_readfirstlane(find_table(p.offsets, p.num_tables, seg_base));
    d = uniform(view(p.descs[f]));
    return f == p.num_tables - 1 || uniform64(seg_base) + seg_len <= uniform64(p.offsets[f + 1]);
}

// ------------------------------------------------------------------ allocation
// TTL test of Sec. 3.4 on a slot that holds an id
__device__ __forceinline__ bool expired(const Tab &d, int32_t step, int64_t s)
{
    return is_expired(d.evict, d.ttl, step, *meta_at(d, s));
}

// One workgroup = one wavefront.  Lane phase: the first PMAX slots of the windows (identities and
// metadata) of up to 64 claimants are read cooperatively -- G lanes read G consecutive slots of
// one claimant with one coalesced access, all accesses in flight together -- and transposed
// through LDS so that every lane then walks the window of its own claimant.  Wave phase: the few
// claimants that go on -- displaced by a better claim, or without a claimable slot among their
// first PMAX -- are served one after the other by the whole wavefront, 64 slots per access.
// The round at which a lane's own claimant was placed is left as a hint for k_finalize.
constexpr uint32_t kHintNone = 0xFF;       // not an elected position
constexpr uint32_t kHintUnplaced = 0xFE;   // ran out of slots: falls back to home (final)
constexpr uint32_t kHintUnknown = 0xFD;    // placed, but not at a round that fits the hint: search the window

// Deferred acceptance by the whole wavefront for the claimant at batch position cpos from round
// cr on (all arguments wave-uniform).  A claimant it displaces is carried on in turn.  Returns
// the round at which the FIRST claimant was placed, or -1 if it ran out of slots.
__device__ __forceinline__ int32_t claim_wave(const Params &p, const Tab &d, uint32_t cpos, int32_t cr)
{
    const int lane = lane_id();
    int64_t home = home_slot(p.ids[cpos], d.seed, d.N);
    int32_t first_round = -1;
    bool is_first = true, active = cr < d.P;
    while (active) {
        // lanes look at rounds cr .. cr + 63
        const int32_t round = cr + lane;
        bool cand = false;
        uint32_t occ = 0;
        int64_t s = 0;
        if (round < d.P) {
            s = wrap(home + round, d.N);
            const int64_t v = __hip_atomic_load(id_at(d, s), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v == -1) cand = true;
            else if (v >= 0) { cand = expired(d, p.step, s); occ = 1; }
            else { occ = tag_occ(v); cand = v > make_tag((uint32_t)round, cpos, occ); }
        }
        uint64_t cmask = __ballot(cand);
        bool placed = false;
        int64_t displaced = 0;
        int32_t placed_round = -1;
        while (cmask && !placed) {
            const int first = __ffsll((unsigned long long)cmask) - 1;
            cmask &= cmask - 1;
            int64_t old = 0, mine = 0;
            if (lane == first) {
                mine = make_tag((uint32_t)round, cpos, occ);
                old = __hip_atomic_fetch_min(id_at(d, s), mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            old = shfl64(old, first);
            mine = shfl64(mine, first);
            if (is_tag(old) && old < mine) continue;          // a better claim got there first
            placed = true;
            placed_round = cr + first;
            displaced = is_tag(old) ? old : 0;
        }
        if (placed) {
            if (is_first) first_round = placed_round;
            is_first = false;
            if (displaced) {
                // carry the displaced claimant on from its next round (same table: same slot)
                cpos = tag_pos(displaced);
                cr = (int32_t)tag_round(displaced) + 1;
                home = home_slot(p.ids[cpos], d.seed, d.N);
                if (cr >= d.P) active = false;                // out of rounds: falls back at finalize
            } else {
                active = false;
            }
        } else {
            cr += kWave;
            if (cr >= d.P) active = false;                    // window exhausted: falls back at finalize
        }
    }
    return first_round;
}

// What the lanes that load a claimant's window need of the claimant's table (several tables only)
struct TabWords {
    int64_t I, M, N;
    int32_t P, ttl, evict, sh;
};

// One wavefront serves the segments vblock, vblock + vgrid, ...; s_I and s_d are that wavefront's own
// areas of LDS (s_d only with several tables).  The lane phase looks at the window in stages of 8
// slots (64 bytes of identities; one 128-byte line of records): nearly every claimant of a table with
// room, or with expired ids, is placed among the first 8, and the second stage is loaded only when a
// lane of the wavefront still needs it.
constexpr int kAllocG = 8;                           // lanes that read one stage of one claimant's window together

template <int PMAX, bool MULTI>
__device__ __forceinline__ void allocate_body(const Params &p, int64_t vblock, int64_t vgrid,
                                              int64_t (*s_I)[kAllocG + 1], TabWords *s_d)
{
    constexpr int G = kAllocG;
    constexpr int APL = kWave / G;                   // claimants served by one load instruction
    constexpr int NT = kWave / APL;                  // load instructions per stage
    constexpr int STAGES = PMAX / G;
    static_assert(PMAX % G == 0, "the lane phase works in stages of 8 slots");

    const int lane = lane_id();
    const int g = lane / G, r = lane % G;
    const Tab d0 = view(p.t0);
    for (int64_t seg = vblock; seg < p.num_segs; seg += vgrid) {
        const uint32_t cnt = p.seg_cnt[seg];
        const int64_t seg_base = seg * p.seg_chunks * kWave;
        if (seg_base >= p.n) break;                           // segments past the batch hold nothing
        int seg_f = 0;
        Tab seg_d = d0;
        bool seg_one = true;
        if constexpr (MULTI) seg_one = segment_table(p, seg_base, p.seg_chunks * kWave, seg_f, seg_d);
        for (uint32_t j0 = 0;; j0 += kWave) {
            // the list entries are requested before the count is known: the count is at most the
            // number of positions of the segment and the arrays have room for n + 128 entries, so
            // the addresses are valid whatever the count turns out to be
            const int64_t idx = seg_base + j0 + lane;
            const uint32_t pos = p.list[idx];
            const uint32_t e = p.ent[idx];
            int64_t home = p.homes[idx];
            if (j0 >= cnt) break;
            const bool have = j0 + lane < cnt;
            bool agent = false;
            int f = 0;
            Tab d = d0;
            if (have) {
                const uint32_t first = p.set_slot[e];
                p.first_of[idx] = first;
                agent = first == pos;                         // else: a later copy of the id
                if (MULTI && agent) {
                    if (seg_one) {
                        f = seg_f;
                        d = seg_d;
                    } else {
                        f = find_table(p.offsets, p.num_tables, (int64_t)pos);
                        d = view(p.descs[f]);
                    }
                    if (d.evict == 2) agent = false;          // claimants of LRU tables are served by k_allocate_lru
                }
            }
            if (!agent) home = 0;
            if constexpr (MULTI) {
                s_d[lane] = TabWords{(int64_t)d.I, (int64_t)d.M, d.N, d.P, d.ttl, d.evict, d.sh};
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            }
            uint32_t hint = agent ? kHintUnplaced : kHintNone;
            bool placed = false;
            bool more = false;           // a claimant of this lane goes on in the wave phase
            uint32_t mpos = 0;
            int32_t mr = 0;
#pragma unroll
            for (int st = 0; st < STAGES; ++st) {
                const int kb = st * G;
                const bool need = agent && !placed && kb < d.P;
                if (st > 0 && !__any(need)) break;
                // cooperative loads of slots kb .. kb + 7 of every claimant that goes on; lanes without
                // a slot to read use the home slot / slot 0 (valid addresses)
                int64_t vi[NT];
                int32_t vm[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int a = t * APL + g;
                    const int64_t ghome = shfl64(home, a);
                    const bool gneed = __shfl((int)need, a) != 0;
                    global_ptr<int64_t> gI = d0.I;
                    global_ptr<int32_t> gM = d0.M;
                    int64_t gN = d0.N;
                    int gP = d0.P, gsh = d0.sh;
                    if constexpr (MULTI) {
                        const TabWords &gd = s_d[a];
                        gI = (global_ptr<int64_t>)gd.I;
                        gM = (global_ptr<int32_t>)gd.M;
                        gN = gd.N;
                        gP = gd.P;
                        gsh = gd.sh;
                    }
                    const int k = kb + r;
                    const int64_t sl = (gneed && k < gP) ? wrap(ghome + k, gN) : ghome;
                    vi[t] = __hip_atomic_load(gI + (sl << gsh), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    vm[t] = gM[sl << (2 * gsh)];
                }
                // what a lane needs to know of a slot: -1 empty, a claim tag (<= -2), 1 = holds an expired
                // id, 0 = holds a live id
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    int32_t gttl = d0.ttl, gev = d0.evict;        // the claimant's table: ttl and eviction mode
                    if constexpr (MULTI) {
                        gttl = s_d[t * APL + g].ttl;
                        gev = s_d[t * APL + g].evict;
                    }
                    int64_t w = vi[t];
                    if (w >= 0) w = is_expired(gev, gttl, p.step, vm[t]) ? 1 : 0;
                    s_I[t * APL + g][r] = w;
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                // lane phase: every lane walks this stage of its own claimant's window
                if (need) {
                    const int lim = d.P < kb + G ? d.P : kb + G;
                    for (int k = kb; k < lim; ++k) {
                        const int64_t v = s_I[lane][k - kb];
                        uint32_t occ = 0;
                        bool cand;
                        if (v == -1) cand = true;
                        else if (v >= 0) { cand = v == 1; occ = 1; }
                        else { occ = tag_occ(v); cand = v > make_tag((uint32_t)k, pos, occ); }
                        if (!cand) continue;
                        const int64_t mine = make_tag((uint32_t)k, pos, occ);
                        const int64_t old = __hip_atomic_fetch_min(id_at(d, wrap(home + k, d.N)), mine, __ATOMIC_RELAXED,
                                                                   __HIP_MEMORY_SCOPE_AGENT);
                        if (is_tag(old) && old < mine) continue;      // a better claim got there first
                        hint = (uint32_t)k;
                        placed = true;
                        if (is_tag(old) && (int32_t)tag_round(old) + 1 < d.P) {
                            // the displaced claimant goes on from its next round (same table: same slot)
                            more = true;
                            mpos = tag_pos(old);
                            mr = (int32_t)tag_round(old) + 1;
                        }
                        break;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // s_I is rewritten by the next stage
            }
            if (agent && !placed && d.P > PMAX) { more = true; mpos = pos; mr = PMAX; }
            // wave phase
            uint64_t lm = __ballot(more);
            while (lm) {
                const int src = __ffsll((unsigned long long)lm) - 1;
                lm &= lm - 1;
                const uint32_t cpos = __shfl(mpos, src);
                const int32_t cr = __shfl(mr, src);
                const uint32_t own = __shfl(pos, src);
                const Tab dw = MULTI ? view(p.descs[__shfl(f, src)]) : d0;
                const int32_t fr = claim_wave(p, dw, cpos, cr);
                if (lane == src && cpos == own)
                    hint = fr < 0 ? kHintUnplaced : (fr < (int32_t)kHintUnknown ? (uint32_t)fr : kHintUnknown);
            }
            if (agent) p.hint[pos] = (uint8_t)hint;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
    }
}

// (+1 column in s_I: rows fall into different banks.)
template <int PMAX, bool MULTI>
__global__ __launch_bounds__(kWave) void k_allocate(Params p)
{
    __shared__ int64_t s_I[kWave][kAllocG + 1];
    __shared__ TabWords s_d[MULTI ? kWave : 1];      // every lane's table, for the lanes that load for it
    allocate_body<PMAX, MULTI>(p, blockIdx.x, gridDim.x, s_I, s_d);
}

// ------------------------------------------------------------------ allocation, LRU policy
// LRU (Sec. 3.4, last paragraph): a missed id takes the first empty slot of its range, else it
// evicts the entry with the oldest time stamp (ties: the earlier probe round), never one seen at
// the current step.  Its preference list -- empty slots in probe order, then evictable slots
// oldest first -- follows from the state at the start of allocation, which stays readable while
// claims are in flight: a tag keeps the was-occupied bit and metadata is not written before
// k_finalize.  The tag's round field carries the CHOICE number, so a slot ends with the claimant
// of the lowest (choice, position).  A group of G lanes serves one claimant, one lane per slot of
// its window (max_probe <= G <= 64; longer ranges: claim_wave_lru_long), so a wavefront works on
// 64 / G claimants at a time; a
// displaced claimant is carried on by the group that displaced it, from its next choice.
// active, cpos and choice are uniform within a group.  Returns the probe round at which the
// group's first claimant was placed, or -1.
template <int G>
__device__ __forceinline__ int32_t claim_group_lru(const Params &p, const Tab &d, bool active, uint32_t cpos,
                                                   int32_t choice)
{
    const int lane = lane_id();
    const int r = lane % G, gbase = lane - r;
    const uint64_t gmask = G == kWave ? ~0ull : ((1ull << (G % kWave)) - 1ull) << gbase;
    const uint64_t below = (1ull << lane) - 1ull;
    int32_t first_round = -1;
    bool is_first = true;
    while (__any(active)) {
        const bool in = active && r < d.P;
        int64_t s = 0, v = 0;
        int32_t m = 0;
        if (in) {
            s = wrap(home_slot(p.ids[cpos], d.seed, d.N) + r, d.N);
            v = __hip_atomic_load(id_at(d, s), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            m = *meta_at(d, s);
        }
        const bool base_empty = in && (v == -1 || (is_tag(v) && !tag_occ(v)));
        const bool evictable = in && (v >= 0 || (is_tag(v) && tag_occ(v))) && m != p.step;
        const uint64_t emask = __ballot(base_empty) & gmask;
        const uint64_t vmask = __ballot(evictable) & gmask;
        const int n_empty = __popcll(emask);
        // rank of this lane's slot in the claimant's preference list
        int older = 0;
        for (int l = 0; l < G; ++l) {
            const int32_t ml = __shfl(m, gbase + l);
            const bool el = (vmask >> (gbase + l)) & 1ull;
            if (el && (ml < m || (ml == m && l < r))) ++older;
        }
        int rank = 0x7FFFFFFF;
        if (base_empty) rank = __popcll(emask & below);
        else if (evictable) rank = n_empty + older;
        const int n_choices = n_empty + __popcll(vmask);
        bool placed = false;
        int64_t displaced = 0;
        bool trying = active && choice < n_choices;
        while (__any(trying)) {
            const uint64_t wb = __ballot(trying && rank == choice) & gmask;
            const int who = __ffsll((unsigned long long)wb) - 1;      // exactly one lane of a trying group has this rank
            int64_t old = 0, mine = 0;
            if (lane == who) {
                mine = make_tag((uint32_t)choice, cpos, base_empty ? 0u : 1u);
                old = __hip_atomic_fetch_min(id_at(d, s), mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const int from = who >= 0 ? who : lane;
            old = shfl64(old, from);
            mine = shfl64(mine, from);
            if (trying) {
                if (is_tag(old) && old < mine) {
                    ++choice;                                           // a better claim holds this slot
                    trying = choice < n_choices;
                } else {
                    placed = true;
                    displaced = is_tag(old) ? old : 0;
                    if (is_first) first_round = who - gbase;
                    trying = false;
                }
            }
        }
        is_first = false;
        if (active) {
            if (!placed || !displaced) {
                active = false;
            } else {
                cpos = tag_pos(displaced);                               // same table: same slot
                choice = (int32_t)tag_round(displaced) + 1;
            }
        }
    }
    return first_round;
}

// One workgroup = one wavefront.  With several tables this kernel runs after k_allocate, which has
// written the hints of every list entry and skipped the claimants of LRU tables; here only those
// claimants are served and only their hints are written.
template <int G, bool MULTI>
__global__ __launch_bounds__(kWave) void k_allocate_lru(Params p)
{
    constexpr int NG = kWave / G;
    const int lane = threadIdx.x;
    const int g = lane / G;
    const Tab d0 = view(MULTI ? p.descs[0] : p.t0);
    for (int64_t seg = blockIdx.x; seg < p.num_segs; seg += gridDim.x) {
        const uint32_t cnt = p.seg_cnt[seg];
        const int64_t seg_base = seg * p.seg_chunks * kWave;
        if (seg_base >= p.n) break;
        for (uint32_t j0 = 0; j0 < cnt; j0 += kWave) {
            const int64_t idx = seg_base + j0 + lane;
            const bool have = j0 + lane < cnt;
            uint32_t pos = 0, e = 0;
            bool agent = false;
            int f = 0;
            if (have) {
                pos = p.list[idx];
                e = p.ent[idx];
                const uint32_t first = p.set_slot[e];
                p.first_of[idx] = first;
                agent = first == pos;
                if (MULTI && agent) {
                    f = find_table(p.offsets, p.num_tables, (int64_t)pos);
                    agent = p.descs[f].evict == 2;
                }
            }
            uint32_t hint = kHintNone;
            uint64_t am = __ballot(agent);
            while (am) {
                // the next NG claimants, one per group of lanes
                int src = -1;
#pragma unroll
                for (int k = 0; k < NG; ++k) {
                    const int sk = am ? __ffsll((unsigned long long)am) - 1 : -1;
                    am &= am - 1;                                         // 0 stays 0
                    if (k == g) src = sk;
                }
                const uint32_t cpos = __shfl(pos, src >= 0 ? src : lane);
                const int fs = __shfl(f, src >= 0 ? src : lane);
                const Tab d = (MULTI && src >= 0) ? view(p.descs[fs]) : d0;
                const int32_t fr = claim_group_lru<G>(p, d, src >= 0, cpos, 0);
                // the outcome goes to the lane that holds the claimant's list entry
#pragma unroll
                for (int k = 0; k < NG; ++k) {
                    const int sk = __shfl(src, k * G);
                    const int32_t frk = __shfl(fr, k * G);
                    if (lane == sk) hint = frk < 0 ? kHintUnplaced : (uint32_t)frk;
                }
            }
            if (agent) p.hint[pos] = (uint8_t)hint;
        }
    }
}

// LRU for probe ranges of 65 .. 1 024 slots: the whole wavefront serves one claimant, a lane holds
// the slots of rounds lane, lane + 64, ...  The preference list is not materialised: choice k is
// the k-th empty slot in probe order while k < number of empty slots, else the (k - empties)-th
// evictable slot in (time stamp, round) order, drawn by repeated wavefront-wide minimum of the
// keys above the previous draw.  Same outcome rule as claim_group_lru.
constexpr int kLruLongSlots = 16;          // slots per lane
constexpr int kLruLongProbe = kLruLongSlots * kWave;

__device__ __forceinline__ uint64_t wave_min64(uint64_t x)
{
    const int lane = lane_id();
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t y = (uint64_t)shfl64((int64_t)x, (lane + o) & 63);
        x = y < x ? y : x;
    }
    return x;
}

__device__ __forceinline__ int32_t claim_wave_lru_long(const Params &p, const Tab &d, uint32_t cpos, int32_t choice)
{
    const int lane = lane_id();
    const int C = (d.P + kWave - 1) / kWave;             // <= kLruLongSlots (checked when the table is created)
    int32_t first_round = -1;
    bool is_first = true;
    for (;;) {
        const int64_t home = home_slot(p.ids[cpos], d.seed, d.N);
        uint32_t emp = 0, evi = 0;                        // bit c: the slot of round c * 64 + lane is empty / evictable
        int32_t m[kLruLongSlots];
#pragma unroll
        for (int c = 0; c < kLruLongSlots; ++c) {
            const int round = c * kWave + lane;
            const bool in = c < C && round < d.P;
            const int64_t s = in ? wrap(home + round, d.N) : home;      // a valid address either way
            const int64_t v = __hip_atomic_load(id_at(d, s), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            m[c] = *meta_at(d, s);
            const bool be = v == -1 || (is_tag(v) && !tag_occ(v));
            const bool oc = v >= 0 || (is_tag(v) && tag_occ(v));
            if (in && be) emp |= 1u << c;
            if (in && oc && m[c] != p.step) evi |= 1u << c;
        }
        int n_empty = 0, n_evict = 0;
        for (int c = 0; c < C; ++c) {
            n_empty += __popcll(__ballot((emp >> c) & 1u));
            n_evict += __popcll(__ballot((evi >> c) & 1u));
        }
        const int n_choices = n_empty + n_evict;
        bool placed = false;
        int64_t displaced = 0;
        uint64_t prev_key = 0;                            // key of the last evictable slot drawn (keys are >= 1)
        int drawn = 0;                                    // evictable slots drawn so far
        for (; choice < n_choices && !placed; ++choice) {
            int round = -1;
            uint32_t occ = 0;
            if (choice < n_empty) {
                int k = choice;
                for (int c = 0; c < C && round < 0; ++c) {
                    uint64_t mask = __ballot((emp >> c) & 1u);
                    const int pc = __popcll(mask);
                    if (k < pc) {
                        for (int i = 0; i < k; ++i) mask &= mask - 1;
                        round = c * kWave + __ffsll((unsigned long long)mask) - 1;
                    } else {
                        k -= pc;
                    }
                }
            } else {
                const int j = choice - n_empty;
                while (drawn <= j) {
                    uint64_t best = ~0ull;
#pragma unroll
                    for (int c = 0; c < kLruLongSlots; ++c) {
                        const uint64_t key =
                            (((uint64_t)((uint32_t)m[c] ^ 0x80000000u) << 32) | (uint32_t)(c * kWave + lane)) + 1ull;
                        if (((evi >> c) & 1u) && key > prev_key && key < best) best = key;
                    }
                    prev_key = wave_min64(best);
                    ++drawn;
                }
                round = (int)(uint32_t)((prev_key - 1ull) & 0xFFFFFFFFull);
                occ = 1;
            }
            if (round < 0) break;                                        // (cannot happen: choice < n_choices)
            const int who = round % kWave;
            int64_t old = 0, mine = 0;
            if (lane == who) {
                mine = make_tag((uint32_t)choice, cpos, occ);
                old = __hip_atomic_fetch_min(id_at(d, wrap(home + round, d.N)), mine, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
            }
            old = shfl64(old, who);
            mine = shfl64(mine, who);
            if (is_tag(old) && old < mine) continue;                    // a better claim holds this slot
            placed = true;
            displaced = is_tag(old) ? old : 0;
            if (is_first) first_round = round;
        }
        is_first = false;
        if (!placed || !displaced) break;
        cpos = tag_pos(displaced);                                       // same table: same slot
        choice = (int32_t)tag_round(displaced) + 1;
    }
    return first_round;
}

template <bool MULTI>
__global__ __launch_bounds__(kWave) void k_allocate_lru_long(Params p)
{
    const int lane = threadIdx.x;
    const Tab d0 = view(MULTI ? p.descs[0] : p.t0);
    for (int64_t seg = blockIdx.x; seg < p.num_segs; seg += gridDim.x) {
        const uint32_t cnt = p.seg_cnt[seg];
        const int64_t seg_base = seg * p.seg_chunks * kWave;
        if (seg_base >= p.n) break;
        for (uint32_t j0 = 0; j0 < cnt; j0 += kWave) {
            const int64_t idx = seg_base + j0 + lane;
            const bool have = j0 + lane < cnt;
            uint32_t pos = 0, e = 0;
            bool agent = false;
            int f = 0;
            if (have) {
                pos = p.list[idx];
                e = p.ent[idx];
                const uint32_t first = p.set_slot[e];
                p.first_of[idx] = first;
                agent = first == pos;
                if (MULTI && agent) {
                    f = find_table(p.offsets, p.num_tables, (int64_t)pos);
                    agent = p.descs[f].evict == 2;
                }
            }
            uint32_t hint = kHintNone;
            uint64_t am = __ballot(agent);
            while (am) {
                const int src = __ffsll((unsigned long long)am) - 1;
                am &= am - 1;
                const uint32_t cpos = __shfl(pos, src);
                const int fs = __shfl(f, src);
                const Tab d = MULTI ? view(p.descs[fs]) : d0;
                const int32_t fr = claim_wave_lru_long(p, d, cpos, 0);
                if (lane == src)
                    hint = fr < 0 ? kHintUnplaced : (fr < (int32_t)kHintUnknown ? (uint32_t)fr : kHintUnknown);
            }
            if (agent) p.hint[pos] = (uint8_t)hint;
        }
    }
}

// ------------------------------------------------------------------ finalize
// Sec. 3.4, fused with the remap: the rows of the evicted slots that this wavefront has staged (row numbers in
// rows_buf) get their initial value.  A row is written by consecutive lanes, 16 (or 4) bytes each.
template <typename VEC>
__device__ __forceinline__ void reset_rows_wave(const Params &p, const int64_t *rows_buf, int count)
{
    const int lane = lane_id();
    const int C = p.g_chunks;
    const int64_t total = (int64_t)count * C;
    for (int64_t i = lane; i < total; i += kWave) {
        const int k = p.g_shift >= 0 ? (int)(i >> p.g_shift) : (int)(i / C);
        const int c = (int)(i - (int64_t)k * C);
        VEC v = VEC(0);
        if (p.r_init) v = reinterpret_cast<const VEC *>(p.r_init)[c];
        __builtin_nontemporal_store(v, reinterpret_cast<VEC *>(p.r_rows + rows_buf[k] * p.g_stride) + c);
    }
}

__device__ __forceinline__ void reset_staged_rows(const Params &p, const int64_t *rows_buf, int count)
{
    if (!p.r_rows || count == 0) return;
    if (p.g_wide) reset_rows_wave<u32x4>(p, rows_buf, count);
    else reset_rows_wave<uint32_t>(p, rows_buf, count);
}

// Appends the staged evicted slots of one wavefront to table `table`'s list (and resets their rows).
__device__ __forceinline__ void flush_evicted(const Params &p, const int64_t *buf, const int64_t *rows_buf, int &count,
                                              int table)
{
    if (count == 0) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    reset_staged_rows(p, rows_buf, count);
    const int lane = lane_id();
    unsigned long long base = 0;
    if (lane == 0)
        base = p.num_tables > 1 ? atomicAdd(&p.ctl->num_evicted[table], (unsigned long long)count)
                                : atomicAdd(&p.ctl->done, (unsigned long long)count) & kEvictedMask;
    base = (unsigned long long)shfl64((int64_t)base, 0);
    // (separate statements: a choice between the descriptor in the kernel arguments and one in global memory,
    // written as one expression, is compiled into loads through a generic pointer)
    int64_t ev_begin = p.t0.ev_begin, ev_cap = p.t0.ev_cap;
    if (p.num_tables > 1) {
        ev_begin = p.descs[table].ev_begin;
        ev_cap = p.descs[table].ev_cap;
    }
    for (int i = lane; i < count; i += kWave) {
        const int64_t at = (int64_t)base + i;
        if (at < ev_cap) p.out_evicted[ev_begin + at] = buf[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    count = 0;
}

// Book-keeping shared by both forms of k_finalize: counters for one table at a time in
// registers, evicted slots staged per wavefront in LDS.
struct FinalizeState {
    int ev_cnt = 0, ev_table = 0;                       // wave-uniform
    unsigned long long st_ins = 0, st_evi = 0, st_col = 0;
    int st_table = 0;
};

// Called by all lanes of the wavefront.  `done` lanes finished a claimant of table f with
// outcome 0 = insert, 1 = eviction of slot s, 2 = collision.
__device__ __forceinline__ void finalize_account(const Params &p, FinalizeState &fs, int64_t *s_ev_w, int64_t *s_row_w,
                                                 bool done, int outcome, int64_t s, int f, bool want_stats)
{
    const int lane = lane_id();
    if (want_stats) {
        if (p.num_tables > 1) {
            const uint64_t dm = __ballot(done);
            if (dm) {
                const int f0 = __shfl(f, __ffsll((unsigned long long)dm) - 1);
                if (f0 != fs.st_table) {
                    // rare (feature boundary): hand the counters over through atomics
                    if (fs.st_ins) atomicAdd(stat_word(p, fs.st_table, kInserts), fs.st_ins);
                    if (fs.st_evi) atomicAdd(stat_word(p, fs.st_table, kEvictions), fs.st_evi);
                    if (fs.st_col) atomicAdd(stat_word(p, fs.st_table, kCollisions), fs.st_col);
                    fs.st_ins = fs.st_evi = fs.st_col = 0;
                    fs.st_table = f0;
                }
            }
        }
        if (done) {
            if (f != fs.st_table) {
                atomicAdd(stat_word(p, f, outcome == 0 ? kInserts : outcome == 1 ? kEvictions : kCollisions), 1ull);
            } else {
                fs.st_ins += outcome == 0;
                fs.st_evi += outcome == 1;
                fs.st_col += outcome == 2;
            }
        }
    }
    // stage evicted slots in LDS; all entries of the buffer belong to one table
    uint64_t evm = __ballot(done && outcome == 1);
    while (evm) {
        const int tf = __shfl(f, __ffsll((unsigned long long)evm) - 1);
        const bool sel = done && outcome == 1 && f == tf;
        const uint64_t selm = __ballot(sel);
        const int add = __popcll(selm);
        if ((fs.ev_cnt > 0 && tf != fs.ev_table) || fs.ev_cnt + add > kEvBuf)
            flush_evicted(p, s_ev_w, s_row_w, fs.ev_cnt, fs.ev_table);
        fs.ev_table = tf;
        if (sel) {
            const int at = fs.ev_cnt + __popcll(selm & ((1ull << lane) - 1ull));
            s_ev_w[at] = s;
            if (p.r_rows) s_row_w[at] = s >= p.g_num_rows ? s % p.g_num_rows : s;
        }
        fs.ev_cnt += add;
        evm &= ~selm;
    }
}

// End of k_finalize, reached by all threads: the workgroup adds its counters to its copy of the call's
// counters, reserves its part of the evicted list (one reservation when all its wavefronts staged for
// the same table) and reports in; returns true in the workgroup that reported in last.  Everything that
// workgroup will read -- evicted counts and counter copies -- was added with device-scope atomics,
// which are performed where all dies see them; a workgroup waits until its own have been acknowledged
// before it reports in.  (A device-scope release fence here would also write back the die's whole L2,
// once per workgroup.)
__device__ __forceinline__ bool finalize_epilogue(const Params &p, FinalizeState &fs, int64_t (*s_ev)[kEvBuf],
                                                  int64_t (*s_row)[kEvBuf], int *s_cnt, int *s_tab,
                                                  unsigned long long *s_base, bool *s_last,
                                                  unsigned long long (*s_red)[kStatCount], bool want_stats)
{
    const int lane = lane_id(), w = threadIdx.x / kWave;
    const bool multi = p.num_tables > 1;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (lane == 0) { s_cnt[w] = fs.ev_cnt; s_tab[w] = fs.ev_table; }
    __syncthreads();
    int total = 0, before = 0, tab = -1;
    bool same = true;
    for (int i = 0; i < kWavesPerBlock; ++i) {
        if (s_cnt[i] == 0) continue;
        if (tab < 0) tab = s_tab[i];
        else if (s_tab[i] != tab) same = false;
        if (i < w) before += s_cnt[i];
        total += s_cnt[i];
    }
    __syncthreads();                                              // s_tab is used again by block_stat_add
    if (want_stats) {
        const int idx[3] = {kInserts, kEvictions, kCollisions};
        const unsigned long long vals[3] = {fs.st_ins, fs.st_evi, fs.st_col};
        block_stat_add(p, idx, vals, 3, fs.st_table, s_red, s_tab);
    }
    if (multi && total > 0 && !same) flush_evicted(p, s_ev[w], s_row[w], fs.ev_cnt, fs.ev_table);
    const bool reserve = total > 0 && (same || !multi);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long arrived;
        if (multi) {
            // the reservation is acknowledged (its result is used) before the workgroup reports in
            if (reserve) *s_base = atomicAdd(&p.ctl->num_evicted[tab], (unsigned long long)total);
            arrived = atomicAdd(&p.ctl->done, kArriveOne);
        } else {
            arrived = atomicAdd(&p.ctl->done, kArriveOne + (unsigned long long)total);
            *s_base = arrived & kEvictedMask;
        }
        *s_last = (arrived >> kArriveShift) == (unsigned long long)(gridDim.x - 1);
    }
    __syncthreads();
    if (reserve) {
        const int64_t base = (int64_t)*s_base + before;
        int64_t ev_begin = p.t0.ev_begin, ev_cap = p.t0.ev_cap;
        if (multi) {
            ev_begin = p.descs[tab].ev_begin;
            ev_cap = p.descs[tab].ev_cap;
        }
        for (int i = lane; i < fs.ev_cnt; i += kWave)
            if (base + i < ev_cap) p.out_evicted[ev_begin + base + i] = s_ev[w][i];
        reset_staged_rows(p, s_row[w], fs.ev_cnt);
    }
    return *s_last;
}

// Every entry of the miss lists -- the elected position of an id (its agent) and the other copies of
// the id alike -- finds the slot that carries the agent's claim: where k_allocate left it (the hint,
// kept under the agent's batch position, which every copy knows), else by a search of the window by
// the whole wavefront (a claimant displaced after its hint was written).  A copy may find the claim
// tag or, when the agent has been quicker, already the id.  The agent turns the tag into the id,
// writes the metadata and accounts for the outcome; every entry stores its output slot.  Entries
// without a claim fall back to the home slot (Case 3).
__device__ __forceinline__ void finalize_body(const Params &p)
{
    __shared__ int64_t s_ev[kWavesPerBlock][kEvBuf];
    __shared__ int64_t s_row[kWavesPerBlock][kEvBuf];              // fused row reset: the rows of the staged slots
    __shared__ unsigned long long s_red[kWavesPerBlock][kStatCount];
    __shared__ unsigned long long s_bins[kMaxTables][kStatCount];
    __shared__ int s_cnt[kWavesPerBlock];
    __shared__ int s_tab[kWavesPerBlock];
    __shared__ unsigned long long s_base;
    __shared__ bool s_last;

    const int lane = lane_id();
    const int w = threadIdx.x / kWave;
    const int64_t wave_global = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
    const int64_t num_waves = (int64_t)gridDim.x * kWavesPerBlock;
    const bool multi = p.num_tables > 1;
    const bool want_stats = p.out_stats != nullptr;
    FinalizeState fs;

    for (int64_t seg = wave_global; seg < p.num_segs; seg += num_waves) {
        const uint32_t cnt = p.seg_cnt[seg];
        const int64_t seg_base = seg * p.seg_chunks * kWave;
        int seg_f = 0;
        Tab seg_d = view(p.t0);
        bool seg_one = true;
        if (multi && cnt > 0) seg_one = segment_table(p, seg_base, p.seg_chunks * kWave, seg_f, seg_d);
        for (uint32_t j0 = 0; j0 < cnt; j0 += kWave) {
            const bool have = j0 + lane < cnt;
            const int64_t idx = seg_base + j0 + lane;
            bool agent = false;
            uint32_t pos = 0, first = 0, h = kHintUnplaced;
            int outcome = 2, f = 0;
            int64_t s_final = 0, home = 0, id = 0;
            Tab d = view(p.t0);
            int at = -1;
            uint32_t occ = 0;
            // does slot value v carry the claim of the id whose first occurrence is `fst`?
            auto is_claim_of = [](int64_t v, uint32_t fst, int64_t cid) {
                return is_tag(v) ? tag_pos(v) == fst : v == cid;
            };
            bool search = false;
            if (have) {
                pos = p.list[idx];
                first = p.first_of[idx];
                agent = first == pos;
                p.set_slot[p.ent[idx]] = kSetEmpty;            // the scratch set is left empty again
                if (multi) {
                    if (seg_one) {
                        f = seg_f;
                        d = seg_d;
                    } else {
                        f = find_table(p.offsets, p.num_tables, (int64_t)pos);
                        d = view(p.descs[f]);
                    }
                }
                id = p.ids[pos];
                home = p.homes[idx];
                h = p.hint[first];
                if (h < kHintUnknown) {
                    const int64_t v = *id_at(d, wrap(home + (int)h, d.N));
                    if (is_claim_of(v, first, id)) { at = (int)h; occ = tag_occ(v); }
                }
                search = at < 0 && h != kHintUnplaced;
            }
            // the hint did not lead to the claim (the claimant was displaced afterwards): the window is
            // searched; searches are served one after the other by the whole wavefront, 64 slots per access
            uint64_t sm = __ballot(search);
            while (sm) {
                const int src = __ffsll((unsigned long long)sm) - 1;
                sm &= sm - 1;
                const uint32_t cfirst = __shfl(first, src);
                const int64_t cid = shfl64(id, src);
                const int64_t chome = shfl64(home, src);
                Tab dw = view(p.t0);
                if (multi) dw = uniform(view(p.descs[__shfl(f, src)]));
                int found_round = -1;
                uint32_t found_occ = 0;
                for (int32_t c0 = 0; c0 < dw.P && found_round < 0; c0 += kWave) {
                    const int32_t round = c0 + lane;
                    bool mine = false;
                    uint32_t o = 0;
                    if (round < dw.P) {
                        const int64_t v = *id_at(dw, wrap(chome + round, dw.N));
                        mine = is_claim_of(v, cfirst, cid);
                        o = tag_occ(v);
                    }
                    const uint64_t mb = __ballot(mine);
                    if (mb) {
                        const int ml = __ffsll((unsigned long long)mb) - 1;
                        found_round = c0 + ml;
                        found_occ = __shfl(o, ml);
                    }
                }
                if (lane == src) { at = found_round; occ = found_occ; }
            }
            if (have) {
                s_final = at >= 0 ? wrap(home + at, d.N) : home;
                if (agent) {
                    // the claim becomes the id, metadata gets its value (Algorithm 1, Pass 2); without a
                    // claim: Case 3, the home slot's metadata is refreshed.  (The agent always meets its
                    // own tag: nobody else replaces it.)
                    if (at >= 0) {
                        *id_at(d, s_final) = id;
                        outcome = (int)occ;
                    }
                    store_meta(d, s_final, meta_value(p, d, pos));
                } else if (p.ttls && d.evict == 3) {
                    // per-feature retention: a later copy may ask for a later expiry step than the first
                    store_meta(d, s_final, meta_value(p, d, pos));
                }
                p.out_slots[pos] = s_final;
            }
            finalize_account(p, fs, s_ev[w], s_row[w], agent, outcome, s_final, f, want_stats);
        }
    }
    // the workgroup that finishes last publishes the call's counters
    const bool last = finalize_epilogue(p, fs, s_ev, s_row, s_cnt, s_tab, &s_base, &s_last, s_red, want_stats);
    if (last) publish_counters(p, s_bins);
}

__global__ __launch_bounds__(kBlock) void k_finalize(Params p)
{
    finalize_body(p);
}

// ------------------------------------------------------------------ fills and row reset
__global__ __launch_bounds__(kBlock) void k_fill64(long long *dst, int64_t count, long long value)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (int64_t)gridDim.x * kBlock)
        dst[i] = value;
}

// initial state of a table kept as 16-byte records: id = -1, metadata = -1, the unused word 0
__global__ __launch_bounds__(kBlock) void k_init_records(u32x4 *dst, int64_t count)
{
    const u32x4 v = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0u};
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (int64_t)gridDim.x * kBlock)
        dst[i] = v;
}

__global__ __launch_bounds__(kBlock) void k_fill32(int32_t *dst, int64_t count, int32_t value)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (int64_t)gridDim.x * kBlock)
        dst[i] = value;
}

// rows[(slots[k] mod num_rows)] <- init (or zero bits).  One thread per VEC-byte chunk of a row,
// so a row is written by consecutive lanes with full-width stores.

template <typename VEC>
__global__ __launch_bounds__(kBlock) void k_reset_rows(const int64_t *slots, const int64_t *count_dev, int64_t cap,
                                                        char *rows, int64_t num_rows, int32_t chunks_per_row,
                                                        int64_t row_stride_bytes, const VEC *init_row)
{
    int64_t count = *count_dev;
    if (count > cap) count = cap;
    if (count < 0) count = 0;
    const int64_t total = count * chunks_per_row;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t k = i / chunks_per_row;
        const int32_t c = (int32_t)(i - k * chunks_per_row);
        int64_t s = slots[k];
        if (s < 0) continue;
        if (s >= num_rows) s %= num_rows;
        VEC v = VEC(0);
        if (init_row) v = init_row[c];
        VEC *dst = reinterpret_cast<VEC *>(rows + s * row_stride_bytes) + c;
        __builtin_nontemporal_store(v, dst);
    }
}

// rows[(slots[k] mod num_rows)] <- init for several tensors at once (embedding weights and
// optimizer state, Sec. 3.4): one thread per VEC-byte chunk of a row of one tensor.
struct RowsDesc {
    char *rows;
    const void *init_row;
    int64_t num_rows;
    int64_t row_stride_bytes;
    int32_t chunks;          // VEC-sized chunks per row
    int32_t pad_;
};
constexpr int kMaxResetTensors = 4;
struct RowsDescs {
    RowsDesc t[kMaxResetTensors];
    int32_t count;
    int32_t total_chunks;
};

template <typename VEC>
__global__ __launch_bounds__(kBlock) void k_reset_rows_multi(const int64_t *slots, const int64_t *count_dev, int64_t cap,
                                                              RowsDescs ds)
{
    int64_t count = *count_dev;
    if (count > cap) count = cap;
    if (count < 0) count = 0;
    const int64_t total = count * ds.total_chunks;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t k = i / ds.total_chunks;
        int32_t c = (int32_t)(i - k * ds.total_chunks);
        int which = 0;
        while (which + 1 < ds.count && c >= ds.t[which].chunks) { c -= ds.t[which].chunks; ++which; }
        const RowsDesc &t = ds.t[which];
        int64_t s = slots[k];
        if (s < 0) continue;
        if (s >= t.num_rows) s %= t.num_rows;
        VEC v = VEC(0);
        if (t.init_row) v = reinterpret_cast<const VEC *>(t.init_row)[c];
        __builtin_nontemporal_store(v, reinterpret_cast<VEC *>(t.rows + s * t.row_stride_bytes) + c);
    }
}

// Row reset for a group of tables in one launch: table f's evicted slots are
// slots[ev_begin .. ev_begin + min(counts[f], ev_cap)), its rows are reset as in k_reset_rows.
struct JagRows {
    char *rows;               // null: nothing to reset for this table
    const void *init_row;
    int64_t num_rows;
    int64_t row_stride_bytes;
    int64_t ev_begin;
    int64_t ev_cap;
    int32_t chunks;           // 16-byte (wide) or 4-byte chunks per row
    int32_t wide;
};

__global__ __launch_bounds__(kBlock) void k_reset_rows_jagged(const int64_t *slots, const int64_t *counts,
                                                               const JagRows *tables, int num_tables)
{
    for (int f = 0; f < num_tables; ++f) {
        const JagRows t = tables[f];
        if (!t.rows) continue;
        int64_t count = counts[f];
        if (count > t.ev_cap) count = t.ev_cap;
        if (count < 0) count = 0;
        const int64_t total = count * t.chunks;
        for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
            const int64_t k = i / t.chunks;
            const int32_t c = (int32_t)(i - k * t.chunks);
            int64_t s = slots[t.ev_begin + k];
            if (s < 0) continue;
            if (s >= t.num_rows) s %= t.num_rows;
            char *row = t.rows + s * t.row_stride_bytes;
            if (t.wide) {
                u32x4 v = u32x4(0);
                if (t.init_row) v = reinterpret_cast<const u32x4 *>(t.init_row)[c];
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(row) + c);
            } else {
                uint32_t v = 0u;
                if (t.init_row) v = reinterpret_cast<const uint32_t *>(t.init_row)[c];
                __builtin_nontemporal_store(v, reinterpret_cast<uint32_t *>(row) + c);
            }
        }
    }
}

// out[k, :] <- rows[slots[k] mod num_rows, :]   (dense output rows of chunks * sizeof(VEC) bytes)
template <typename VEC>
__global__ __launch_bounds__(kBlock) void k_gather_rows(const int64_t *slots, const int64_t *count_dev, int64_t cap,
                                                         const char *rows, int64_t num_rows, int32_t chunks,
                                                         int64_t row_stride_bytes, VEC *out)
{
    int64_t count = count_dev ? *count_dev : cap;
    if (count > cap) count = cap;
    if (count < 0) count = 0;
    const int64_t total = count * chunks;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t k = i / chunks;
        const int32_t c = (int32_t)(i - k * chunks);
        int64_t s = slots[k];
        VEC v = VEC(0);
        if (s >= 0) {
            if (s >= num_rows) s %= num_rows;
            v = reinterpret_cast<const VEC *>(rows + s * row_stride_bytes)[c];
        }
        out[i] = v;
    }
}

// Streaming delta, receiving side (Sec. 3.8): rows[slots[k] mod num_rows, :] <- delta_rows[k, :] in one launch
// and identities[slots[k]] <- ids[k] in the next one on the same stream, so that every row of the delta
// has landed before any identity points at it (a reader on another stream never finds a new id in
// front of a row that is still partly old).
template <typename VEC>
__global__ __launch_bounds__(kBlock) void k_apply_delta_rows(int64_t num_slots, const int64_t *slots,
                                                              const int64_t *count_dev, int64_t cap,
                                                              char *rows, int64_t num_rows, int32_t chunks,
                                                              int64_t row_stride_bytes, const VEC *delta_rows)
{
    int64_t count = count_dev ? *count_dev : cap;
    if (count > cap) count = cap;
    if (count < 0) count = 0;
    const int64_t total = count * chunks;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t k = i / chunks;
        const int32_t c = (int32_t)(i - k * chunks);
        const int64_t s = slots[k];
        if (s < 0 || s >= num_slots) continue;
        const int64_t r = s >= num_rows ? s % num_rows : s;
        reinterpret_cast<VEC *>(rows + r * row_stride_bytes)[c] = delta_rows[i];
    }
}

__global__ __launch_bounds__(kBlock) void k_apply_delta_ids(int64_t *identities, int64_t num_slots, const int64_t *slots,
                                                             const int64_t *ids, const int64_t *count_dev, int64_t cap)
{
    int64_t count = count_dev ? *count_dev : cap;
    if (count > cap) count = cap;
    if (count < 0) count = 0;
    for (int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x; k < count; k += (int64_t)gridDim.x * kBlock) {
        const int64_t s = slots[k];
        if (s < 0 || s >= num_slots) continue;
        __hip_atomic_store(&identities[s], ids[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Streaming delta, sending side (Sec. 3.8): every occupied slot whose metadata is >= since goes to the
// list (slot, id), order unspecified.  A workgroup scans a contiguous range of slots, stages its finds in
// LDS and appends them with one reservation per kDeltaStage finds.
constexpr int kDeltaStage = 1024;
constexpr int kDeltaPerThread = 4;     // slots a thread looks at between two workgroup barriers

__global__ __launch_bounds__(kBlock) void k_collect_delta(const int64_t *identities, const int32_t *metadata, int sh,
                                                          int64_t num_slots, int32_t since, int64_t *out_slots,
                                                          int64_t *out_ids, int64_t cap, unsigned long long *out_count)
{
    __shared__ int64_t s_slot[kDeltaStage + kDeltaPerThread * kBlock];
    __shared__ int s_n;
    __shared__ unsigned long long s_base;
    const int64_t per_block = (num_slots + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per_block;
    const int64_t hi = lo + per_block < num_slots ? lo + per_block : num_slots;
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    auto flush = [&]() {       // reached by all threads, with the staging complete and s_n at rest
        const int n = s_n;
        if (threadIdx.x == 0 && n) s_base = atomicAdd(out_count, (unsigned long long)n);
        __syncthreads();       // everyone has read s_n and sees s_base
        for (int i = threadIdx.x; i < n; i += kBlock) {
            const int64_t at = (int64_t)s_base + i;
            if (at < cap) { out_slots[at] = s_slot[i]; out_ids[at] = identities[s_slot[i] << sh]; }
        }
        if (threadIdx.x == 0) s_n = 0;
        __syncthreads();       // the staging area is free again before anyone adds to it
    };
    for (int64_t base = lo; base < hi; base += kDeltaPerThread * kBlock) {
#pragma unroll
        for (int k = 0; k < kDeltaPerThread; ++k) {
            const int64_t s = base + k * kBlock + threadIdx.x;
            if (s < hi && identities[s << sh] >= 0 && metadata[s << (2 * sh)] >= since) s_slot[atomicAdd(&s_n, 1)] = s;
        }
        __syncthreads();
        // The decision to flush is taken by all threads from the same value: s_n does not change
        // between the barrier above and the one inside flush (or the one below).
        const bool full = s_n > kDeltaStage;
        if (full) flush();
        else __syncthreads();  // nobody adds to s_n before everyone has looked at it
    }
    flush();
}

}  // namespace mpzch
