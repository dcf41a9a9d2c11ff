// Device code of the MPZCH batched remap for gfx950 (wave64).
//
// Kernel sequence of one training remap (paper Sec. 3.2 / Algorithm 1, Sec. 3.4, Sec. 3.6):
//   k_discover   Pass 1 for every position: a G-lane group loads the probe window of one id
//                with one coalesced access and finds the id by ballot + ffs.  Hits store
//                metadata = step and the output slot; misses go to a compact miss list and
//                into a scratch hash set that elects, per distinct missed id, the position of
//                its first occurrence (input de-duplication of the ids that must allocate).
//   k_allocate   the elected positions claim slots.  A claim is a 64-bit atomic min of a tag
//                (round, first position) into the identities word, so a slot always ends up
//                with the claimant of the lowest (round, position); a claimant that is
//                displaced is carried on by the displacing group from its next round.  The
//                fixed point is the unique stable assignment, the same one a sequential
//                round-major / position-minor sweep produces.
//   k_finalize   every elected id finds its tag in its window, replaces it by the id, sets
//                metadata = step, reports evicted slots; ids without a tag fall back to home.
//   k_emit_dups  the other copies of a missed id copy the slot of the elected position.
//   k_cleanup    re-empties the scratch set entries that were used and publishes counters.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mpzch {

constexpr int kWave = 64;
constexpr int kBlock = 256;
constexpr int kMaxTables = 64;
constexpr int kStatCount = 8;

enum Stat { kHitPos = 0, kMissPos, kDistinctMiss, kInserts, kEvictions, kCollisions, kInvalidPos, kHitProbeSum };

struct TableDesc {
    int64_t *I;            // identities
    int32_t *M;            // metadata (last-seen step)
    int64_t N;             // slots
    uint64_t seed;
    int32_t P;             // min(max_probe, N)
    int32_t ttl;
    int32_t evict;         // 0 = off, 1 = TTL
    int32_t pad_;
    int64_t ev_begin;      // where this table's evicted list starts in out_evicted
    int64_t ev_cap;
};

// Counters of one call.  Two copies exist; a call uses one and zeroes the other for the next call.
struct Control {
    unsigned long long miss_count;
    unsigned long long pad_[7];
    unsigned long long num_evicted[kMaxTables];
    unsigned long long stats[kMaxTables][kStatCount];
};

struct Params {
    const int64_t *ids;
    int64_t n;
    int32_t step;
    int32_t num_tables;            // 1 => t0 is used and offsets/descs are ignored
    int64_t *out_slots;
    uint8_t *out_found;            // lookup only, may be null
    // scratch
    uint32_t *miss_pos;
    uint32_t *miss_ent;
    long long *set_keys;           // scratch hash set: key = id, empty = -1
    uint32_t *set_minpos;          // smallest position that inserted the key, empty = 0xFFFFFFFF
    Control *ctl;
    Control *ctl_next;
    // several tables
    const TableDesc *descs;        // device array [num_tables]
    const int64_t *offsets;        // device array [num_tables + 1]
    TableDesc t0;
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

template <int G>
__device__ __forceinline__ uint32_t group_bits(uint64_t ballot, int group)
{
    if constexpr (G == 64) return 0;  // not used: see group_bits64
    return (uint32_t)(ballot >> (group * G)) & (uint32_t)((1ull << G) - 1ull);
}

// first set bit (0-based) of this group's part of a ballot, or -1
template <int G>
__device__ __forceinline__ int group_first(uint64_t ballot, int group)
{
    if constexpr (G == 64) {
        return ballot ? __ffsll((unsigned long long)ballot) - 1 : -1;
    } else {
        uint32_t b = group_bits<G>(ballot, group);
        return b ? __ffs(b) - 1 : -1;
    }
}

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

// ------------------------------------------------------------------ scratch set
constexpr uint64_t kSetSeed = 0x2545F4914F6CDD1Dull;

// Inserts (id -> min position) into the region [base, base + size) of the scratch set and
// returns the entry index.  size >= 2 * (number of inserts into the region), so the unbounded
// probe always ends.
__device__ __forceinline__ uint32_t set_insert(const Params &p, int64_t id, uint32_t pos, uint64_t base, uint64_t size)
{
    uint64_t e = base + __umul64hi(mix64((uint64_t)id ^ kSetSeed), size);
    const uint64_t end = base + size;
    for (;;) {
        long long k = __hip_atomic_load(&p.set_keys[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (k == -1) {
            long long expected = -1;
            if (__hip_atomic_compare_exchange_strong(&p.set_keys[e], &expected, (long long)id, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                break;
            k = expected;
        }
        if (k == (long long)id) break;
        if (++e == end) e = base;
    }
    __hip_atomic_fetch_min(&p.set_minpos[e], pos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return (uint32_t)e;
}

// ------------------------------------------------------------------ Pass 1 (discovery)
// Probes the windows of the 64 ids held one per lane.  d is wave-uniform.  `on` marks lanes
// whose id is valid and belongs to table d.  Returns, per lane, the probe distance of the hit
// or -1.  A group of G lanes loads G consecutive slots per access; 64 / G ids per access.
template <int G>
__device__ __forceinline__ int probe_wave(const TableDesc &d, int64_t id, int64_t home, bool on)
{
    constexpr int IPI = kWave / G;           // ids per iteration
    const int lane = lane_id();
    const int g = lane / G, r = lane % G;
    int my_dist = -1;
    if (d.P <= G) {
#pragma unroll
        for (int t = 0; t < G; ++t) {
            const int src = t * IPI + g;
            const int64_t gid = shfl64(id, src);
            const int64_t ghome = shfl64(home, src);
            const bool act = __shfl((int)on, src) && r < d.P;
            int64_t v = -1;
            if (act) v = d.I[wrap(ghome + r, d.N)];
            const uint64_t b = __ballot(act && v == gid);
            const int first = group_first<G>(b, g);
            const int got = __shfl(first, (lane % IPI) * G);
            if (lane / IPI == t) my_dist = got;
        }
    } else {
        // window longer than a group: scan it in chunks of G, stop at the first match
        for (int t = 0; t < G; ++t) {
            const int src = t * IPI + g;
            const int64_t gid = shfl64(id, src);
            const int64_t ghome = shfl64(home, src);
            const bool gon = __shfl((int)on, src);
            int first = -1;
            for (int c = 0; c < d.P; c += G) {
                const bool act = gon && first < 0 && (c + r) < d.P;
                int64_t v = -1;
                if (act) {
                    int64_t s = ghome + c + r;          // home < N, c + r < P <= N
                    v = d.I[wrap(s, d.N)];
                }
                const uint64_t b = __ballot(act && v == gid);
                const int f = group_first<G>(b, g);
                if (first < 0 && f >= 0) first = c + f;
                if (__all(first >= 0 || !gon)) break;
            }
            const int got = __shfl(first, (lane % IPI) * G);
            if (lane / IPI == t) my_dist = got;
        }
    }
    return my_dist;
}

template <int G, bool TRAIN>
__global__ __launch_bounds__(kBlock) void k_discover(Params p)
{
    const int lane = lane_id();
    const int64_t wave_global = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
    const int64_t num_waves = (int64_t)gridDim.x * (kBlock / kWave);
    const bool multi = p.num_tables > 1;

    if (TRAIN && blockIdx.x == 0) {
        // zero the other counter block for the next call
        unsigned long long *z = reinterpret_cast<unsigned long long *>(p.ctl_next);
        for (int i = threadIdx.x; i < (int)(sizeof(Control) / sizeof(unsigned long long)); i += kBlock) z[i] = 0ull;
    }

    // per-lane statistics of the table currently being processed
    unsigned long long st_hit = 0, st_miss = 0, st_inv = 0, st_probe = 0;
    int st_table = 0;
    auto flush_stats = [&]() {
        if (!TRAIN) return;
        unsigned long long v[4] = {st_hit, st_miss, st_inv, st_probe};
        const int idx[4] = {kHitPos, kMissPos, kInvalidPos, kHitProbeSum};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            unsigned long long x = v[k];
            for (int o = 32; o > 0; o >>= 1) x += (unsigned long long)shfl64((int64_t)x, (lane + o) & 63);
            // after the rotation-sum every lane holds the wave total
            if (lane == 0 && x) atomicAdd(&p.ctl->stats[st_table][idx[k]], x);
        }
        st_hit = st_miss = st_inv = st_probe = 0;
    };

    for (int64_t base = wave_global * kWave; base < p.n; base += num_waves * kWave) {
        const int64_t pos = base + lane;
        const bool in_range = pos < p.n;
        const int64_t id = in_range ? p.ids[pos] : -1;
        bool todo = in_range;
        // every pass handles the lanes that belong to one table (one pass unless the wave
        // straddles a feature boundary)
        while (__any(todo)) {
            TableDesc d;
            int f = 0;
            uint64_t set_base = 0, set_size = 2ull * (uint64_t)p.n;
            bool mine = todo;
            if (multi) {
                const uint64_t tb = __ballot(todo);
                const int first_lane = __ffsll((unsigned long long)tb) - 1;
                const int64_t first_pos = base + first_lane;
                f = find_table(p.offsets, p.num_tables, first_pos);
                f = __builtin_amdgcn_readfirstlane(f);
                // find_table skips empty features that share this offset.  The clamps keep every
                // access in bounds (and the loop finite) even if the offsets break their contract.
                int64_t seg_lo = p.offsets[f], seg_hi = p.offsets[f + 1];
                if (f == p.num_tables - 1 || seg_hi > p.n) seg_hi = p.n;
                if (seg_hi <= first_pos) seg_hi = first_pos + 1;
                if (seg_lo > first_pos) seg_lo = first_pos;
                if (seg_lo < 0) seg_lo = 0;
                d = p.descs[f];
                mine = todo && pos < seg_hi;
                set_base = 2ull * (uint64_t)seg_lo;
                set_size = 2ull * (uint64_t)(seg_hi - seg_lo);
            } else {
                d = p.t0;
            }
            if (TRAIN && f != st_table) { flush_stats(); st_table = f; }

            const bool valid = mine && id >= 0;
            const int64_t home = mine ? home_slot(id, d.seed, d.N) : 0;
            const int dist = probe_wave<G>(d, id, home, valid);
            const bool hit = valid && dist >= 0;
            const int64_t slot = hit ? wrap(home + dist, d.N) : home;

            if (TRAIN) {
                if (hit) {
                    d.M[slot] = p.step;                   // "Update": refresh the resident's metadata
                    p.out_slots[pos] = slot;
                    st_hit++;
                    st_probe += (unsigned long long)(dist + 1);
                } else if (mine && !valid) {
                    p.out_slots[pos] = slot;               // negative id: home of its bit pattern
                    st_inv++;
                }
                const bool miss = valid && !hit;
                const uint64_t mb = __ballot(miss);
                if (mb) {
                    uint32_t start = 0;
                    const int leader = __ffsll((unsigned long long)mb) - 1;
                    if (lane == leader)
                        start = (uint32_t)atomicAdd(&p.ctl->miss_count, (unsigned long long)__popcll(mb));
                    start = __shfl(start, leader);
                    if (miss) {
                        const uint32_t k = start + (uint32_t)__popcll(mb & ((1ull << lane) - 1ull));
                        p.miss_pos[k] = (uint32_t)pos;
                        p.miss_ent[k] = set_insert(p, id, (uint32_t)pos, set_base, set_size);
                        st_miss++;
                    }
                }
            } else {
                if (mine) {
                    p.out_slots[pos] = slot;
                    if (p.out_found) p.out_found[pos] = hit ? 1 : 0;
                }
            }
            todo = todo && !mine;
        }
    }
    flush_stats();
}

// ------------------------------------------------------------------ allocation
// One G-lane group per entry of the miss list.  The group of the elected position of an id
// runs deferred acceptance for it: propose to the first slot of the window that is claimable
// and not held by a better tag; on displacing another tag continue on behalf of its owner.
template <int G>
__global__ __launch_bounds__(kBlock) void k_allocate(Params p)
{
    constexpr int GPW = kWave / G;  // groups per wave
    const int lane = lane_id();
    const int g = lane / G, r = lane % G;
    const int64_t wave_global = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
    const int64_t num_waves = (int64_t)gridDim.x * (kBlock / kWave);
    const unsigned long long n_miss = p.ctl->miss_count;
    const bool multi = p.num_tables > 1;

    for (uint64_t kb = (uint64_t)wave_global * GPW; kb < n_miss; kb += (uint64_t)num_waves * GPW) {
        const uint64_t k = kb + g;
        // group-uniform state of the claimant carried by this group
        bool active = false;
        uint32_t cpos = 0;      // its position (priority within a round)
        int64_t cid = 0;        // its id
        int32_t cr = 0;         // next round to try
        TableDesc d = p.t0;
        int64_t home = 0;
        if (k < n_miss) {
            cpos = p.miss_pos[k];
            const uint32_t e = p.miss_ent[k];
            active = (p.set_minpos[e] == cpos);   // elected: first occurrence of its id
            if (active) {
                cid = p.ids[cpos];
                int f = 0;
                if (multi) { f = find_table(p.offsets, p.num_tables, (int64_t)cpos); d = p.descs[f]; }
                home = home_slot(cid, d.seed, d.N);
                if (r == 0) atomicAdd(&p.ctl->stats[f][kDistinctMiss], 1ull);
            }
        }
        while (__any(active)) {
            // scan rounds cr + r of the claimant's window
            const int32_t round = cr + r;
            const bool inr = active && round < d.P;
            bool cand = false;
            uint32_t occ = 0;
            int64_t s = 0;
            if (inr) {
                s = wrap(home + round, d.N);
                const int64_t v = __hip_atomic_load(&d.I[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v == -1) {
                    cand = true;
                } else if (v >= 0) {
                    if (d.evict && (int64_t)p.step - (int64_t)d.M[s] > (int64_t)d.ttl) { cand = true; occ = 1; }
                } else {
                    occ = tag_occ(v);
                    cand = v > make_tag((uint32_t)round, cpos, occ);   // held by a worse claim
                }
            }
            uint64_t cmask = __ballot(cand);
            // propose to candidates in probe order until one accepts
            bool settled = !active;     // this group is done with the current scan
            bool placed = false;
            int64_t displaced = 0;      // tag that was displaced (0 = none)
            while (true) {
                const int first = settled ? -1 : group_first<G>(cmask, g);
                if (!settled && first < 0) settled = true;        // no candidate left in this scan
                if (__all(settled)) break;
                int64_t old = 0;
                if (!settled && r == first) {
                    const int64_t mine = make_tag((uint32_t)round, cpos, occ);
                    old = __hip_atomic_fetch_min(&d.I[s], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (!settled) {
                    old = shfl64(old, g * G + first);
                    const int64_t mine_first = make_tag((uint32_t)(cr + first), cpos, tag_occ(old));
                    if (is_tag(old) && old < mine_first) {
                        // a better claim got there first: this slot is lost for good
                        if constexpr (G == 64) cmask &= ~(1ull << first);
                        else cmask &= ~(1ull << (g * G + first));
                    } else {
                        placed = true;
                        settled = true;
                        displaced = is_tag(old) ? old : 0;
                    }
                }
            }
            if (active) {
                if (placed) {
                    if (displaced) {
                        // carry the displaced claimant on from its next round
                        cpos = tag_pos(displaced);
                        cr = (int32_t)tag_round(displaced) + 1;
                        cid = p.ids[cpos];
                        // same table: both claimed the same slot
                        home = home_slot(cid, d.seed, d.N);
                        if (cr >= d.P) active = false;       // out of rounds: falls back at finalize
                    } else {
                        active = false;
                    }
                } else {
                    cr += G;
                    if (cr >= d.P) active = false;           // window exhausted: falls back at finalize
                }
            }
        }
    }
}

// ------------------------------------------------------------------ finalize
template <int G>
__global__ __launch_bounds__(kBlock) void k_finalize(Params p)
{
    constexpr int GPW = kWave / G;
    const int lane = lane_id();
    const int g = lane / G, r = lane % G;
    const int64_t wave_global = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
    const int64_t num_waves = (int64_t)gridDim.x * (kBlock / kWave);
    const unsigned long long n_miss = p.ctl->miss_count;
    const bool multi = p.num_tables > 1;

    for (uint64_t kb = (uint64_t)wave_global * GPW; kb < n_miss; kb += (uint64_t)num_waves * GPW) {
        const uint64_t k = kb + g;
        bool active = false;
        uint32_t cpos = 0;
        int64_t cid = 0, home = 0;
        int f = 0;
        TableDesc d = p.t0;
        if (k < n_miss) {
            cpos = p.miss_pos[k];
            active = (p.set_minpos[p.miss_ent[k]] == cpos);
            if (active) {
                cid = p.ids[cpos];
                if (multi) { f = find_table(p.offsets, p.num_tables, (int64_t)cpos); d = p.descs[f]; }
                home = home_slot(cid, d.seed, d.N);
            }
        }
        // find the slot that carries this claimant's tag
        int found = -1;          // round at which it sits
        bool searching = active;
        for (int32_t c = 0; __any(searching); c += G) {
            const int32_t round = c + r;
            const bool inr = searching && round < d.P;
            bool m = false;
            if (inr) {
                const int64_t s = wrap(home + round, d.N);
                const int64_t v = __hip_atomic_load(&d.I[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                m = is_tag(v) && tag_pos(v) == cpos;
                if (m) {
                    // claim becomes the id; metadata gets the step (Algorithm 1, Pass 2)
                    __hip_atomic_store(&d.I[s], cid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    d.M[s] = p.step;
                    p.out_slots[cpos] = s;
                    if (tag_occ(v)) {
                        const unsigned long long at = atomicAdd(&p.ctl->num_evicted[f], 1ull);
                        if ((int64_t)at < d.ev_cap) p.out_evicted[d.ev_begin + (int64_t)at] = s;
                        atomicAdd(&p.ctl->stats[f][kEvictions], 1ull);
                    } else {
                        atomicAdd(&p.ctl->stats[f][kInserts], 1ull);
                    }
                }
            }
            const int first = group_first<G>(__ballot(m), g);
            if (searching) {
                if (first >= 0) { found = c + first; searching = false; }
                else if (c + G >= d.P) searching = false;
            }
        }
        if (active && found < 0 && r == 0) {
            // Case 3: no empty or evictable slot -> home slot, its metadata refreshed
            d.M[home] = p.step;
            p.out_slots[cpos] = home;
            atomicAdd(&p.ctl->stats[f][kCollisions], 1ull);
        }
    }
}

// ------------------------------------------------------------------ duplicates + cleanup
__global__ __launch_bounds__(kBlock) void k_emit_dups(Params p)
{
    const unsigned long long n_miss = p.ctl->miss_count;
    for (uint64_t k = (uint64_t)blockIdx.x * kBlock + threadIdx.x; k < n_miss; k += (uint64_t)gridDim.x * kBlock) {
        const uint32_t pos = p.miss_pos[k];
        const uint32_t first = p.set_minpos[p.miss_ent[k]];
        if (first != pos) p.out_slots[pos] = p.out_slots[first];
    }
}

__global__ __launch_bounds__(kBlock) void k_cleanup(Params p)
{
    const unsigned long long n_miss = p.ctl->miss_count;
    for (uint64_t k = (uint64_t)blockIdx.x * kBlock + threadIdx.x; k < n_miss; k += (uint64_t)gridDim.x * kBlock) {
        const uint32_t e = p.miss_ent[k];
        p.set_keys[e] = -1;
        p.set_minpos[e] = 0xFFFFFFFFu;
    }
    if (blockIdx.x == 0) {
        for (int i = threadIdx.x; i < p.num_tables; i += kBlock)
            p.out_num_evicted[i] = (int64_t)p.ctl->num_evicted[i];
        if (p.out_stats)
            for (int i = threadIdx.x; i < p.num_tables * kStatCount; i += kBlock)
                p.out_stats[i] = (int64_t)p.ctl->stats[i / kStatCount][i % kStatCount];
    }
}

// ------------------------------------------------------------------ fills and row reset
__global__ __launch_bounds__(kBlock) void k_fill64(long long *dst, int64_t count, long long value)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (int64_t)gridDim.x * kBlock)
        dst[i] = value;
}

__global__ __launch_bounds__(kBlock) void k_fill32(int32_t *dst, int64_t count, int32_t value)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (int64_t)gridDim.x * kBlock)
        dst[i] = value;
}

// rows[(slots[k] mod num_rows)] <- init (or zero bits).  One thread per VEC-byte chunk of a row,
// so a row is written by consecutive lanes with full-width stores.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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

}  // namespace mpzch
