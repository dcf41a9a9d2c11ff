// Device code of the MPZCH batched remap for gfx950 (wave64).
//
// Kernel sequence of one training remap (paper Sec. 3.2 / Algorithm 1, Sec. 3.4, Sec. 3.6):
//   k_discover   Pass 1 for every position: a G-lane group loads the probe window of one id
//                with one coalesced access and finds the id by ballot + ffs.  Hits store
//                metadata = step and the output slot.  Misses set their bit in a per-64-position
//                miss mask and enter a scratch hash set that elects, per distinct missed id,
//                the position of its first occurrence (input de-duplication of the ids that
//                must allocate).
//   k_allocate   the elected positions claim slots.  A claim is a 64-bit atomic min of a tag
//                (round, first position) into the identities word, so a slot always ends up
//                with the claimant of the lowest (round, position); a claimant that is
//                displaced is carried on by the displacing group from its next round.  The
//                fixed point is the unique stable assignment, the same one a sequential
//                round-major / position-minor sweep produces.
//   k_finalize   every elected id finds its tag in its window, replaces it by the id, sets
//                metadata = step and reports evicted slots; ids without a tag fall back to home.
//   k_emit_dups  the other copies of a missed id copy the slot of the elected position; the
//                scratch set entries that were used are emptied again; counters are published.
//
// No kernel funnels work through one hot address: an atomic on a single address costs about
// 12 ns on this GPU however many lanes it serves, so the miss list is a bit mask per wavefront
// chunk (no shared cursor), counters are accumulated per wavefront and reduced once, and evicted
// slots are staged in LDS and appended with one reservation per workgroup.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mpzch {

constexpr int kWave = 64;
constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxTables = 64;
constexpr int kStatCount = 8;
constexpr int kEvBuf = 256;            // evicted slots staged per wavefront before a flush

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

// Counters of one call that do go through atomics (few per call).  Two copies exist; a call
// uses one and zeroes the other for the next call.
struct Control {
    unsigned long long num_evicted[kMaxTables];
    unsigned long long stats[kMaxTables][kStatCount];
};

// Per-wavefront partial counters, written once with plain stores and summed by k_emit_dups.
struct StatRow {
    unsigned long long v[kStatCount];
    long long table;
};

struct Params {
    const int64_t *ids;
    int64_t n;
    int32_t step;
    int32_t num_tables;            // 1 => t0 is used and offsets/descs are ignored
    int64_t *out_slots;
    uint8_t *out_found;            // lookup only, may be null
    // scratch
    unsigned long long *miss_mask; // word c: which of the positions [64c, 64c + 64) missed
    uint32_t *ent;                 // per miss position: its entry in the scratch set
    uint32_t *first_of;            // per miss position: position of the first occurrence of its id
    long long *set_keys;           // scratch hash set: key = id, empty = -1
    uint32_t *set_minpos;          // smallest position that inserted the key, empty = 0xFFFFFFFF
    StatRow *rows_a;               // per wavefront of k_discover
    StatRow *rows_b;               // per wavefront of k_finalize
    int32_t waves_a, waves_b;
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
    if constexpr (G == 64) return 0;  // a 64-lane group reads the whole ballot, see group_first
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

// contiguous range of 64-position chunks owned by this wavefront
__device__ __forceinline__ void wave_chunk_range(int64_t n, int64_t &c_begin, int64_t &c_end, int64_t &wave_global)
{
    wave_global = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
    const int64_t num_waves = (int64_t)gridDim.x * kWavesPerBlock;
    const int64_t num_chunks = (n + kWave - 1) / kWave;
    const int64_t per_wave = (num_chunks + num_waves - 1) / num_waves;
    c_begin = wave_global * per_wave;
    c_end = c_begin + per_wave < num_chunks ? c_begin + per_wave : num_chunks;
}

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long x)
{
    // rotation sum: afterwards every lane holds the wavefront total
    const int lane = lane_id();
    for (int o = 32; o > 0; o >>= 1) x += (unsigned long long)shfl64((int64_t)x, (lane + o) & 63);
    return x;
}

__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

template <int G, bool TRAIN>
__global__ __launch_bounds__(kBlock) void k_discover(Params p)
{
    const int lane = lane_id();
    int64_t c_begin, c_end, wave_global;
    wave_chunk_range(p.n, c_begin, c_end, wave_global);
    const bool multi = p.num_tables > 1;
    const bool want_stats = TRAIN && p.out_stats != nullptr;

    if (TRAIN && blockIdx.x == 0) {
        // zero the other counter block for the next call
        unsigned long long *z = reinterpret_cast<unsigned long long *>(p.ctl_next);
        for (int i = threadIdx.x; i < (int)(sizeof(Control) / sizeof(unsigned long long)); i += kBlock) z[i] = 0ull;
    }

    // per-lane counters of the table currently being processed
    unsigned long long st_hit = 0, st_miss = 0, st_inv = 0, st_probe = 0;
    int st_table = 0;

    for (int64_t c = c_begin; c < c_end; ++c) {
        const int64_t base = c * kWave;
        const int64_t pos = base + lane;
        const bool in_range = pos < p.n;
        const int64_t id = in_range ? p.ids[pos] : -1;
        bool todo = in_range;
        uint64_t miss_bits = 0;
        // every pass handles the lanes that belong to one table (one pass unless the chunk
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
            if (want_stats && f != st_table) {
                // table changed inside this wavefront's range (rare): hand the counters over
                const unsigned long long a = wave_sum(st_hit), b = wave_sum(st_miss), x = wave_sum(st_inv),
                                         y = wave_sum(st_probe);
                if (lane == 0) {
                    if (a) atomicAdd(&p.ctl->stats[st_table][kHitPos], a);
                    if (b) atomicAdd(&p.ctl->stats[st_table][kMissPos], b);
                    if (x) atomicAdd(&p.ctl->stats[st_table][kInvalidPos], x);
                    if (y) atomicAdd(&p.ctl->stats[st_table][kHitProbeSum], y);
                }
                st_hit = st_miss = st_inv = st_probe = 0;
                st_table = f;
            }

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
                miss_bits |= __ballot(miss);
                if (miss) {
                    p.ent[pos] = set_insert(p, id, (uint32_t)pos, set_base, set_size);
                    st_miss++;
                }
            } else {
                if (mine) {
                    p.out_slots[pos] = slot;
                    if (p.out_found) p.out_found[pos] = hit ? 1 : 0;
                }
            }
            todo = todo && !mine;
        }
        if (TRAIN && lane == 0) p.miss_mask[c] = miss_bits;
    }
    if (want_stats) {
        const unsigned long long a = wave_sum(st_hit), b = wave_sum(st_miss), x = wave_sum(st_inv),
                                 y = wave_sum(st_probe);
        if (lane == 0 && wave_global < p.waves_a) {
            StatRow row;
            for (int k = 0; k < kStatCount; ++k) row.v[k] = 0;
            row.v[kHitPos] = a;
            row.v[kMissPos] = b;
            row.v[kInvalidPos] = x;
            row.v[kHitProbeSum] = y;
            row.table = st_table;
            p.rows_a[wave_global] = row;
        }
    }
}

// ------------------------------------------------------------------ allocation
// Loads, one miss position per lane, what k_allocate / k_finalize need of a 64-position chunk
// and returns the ballot of the elected positions (first occurrence of their id).
template <bool STORE_FIRST>
__device__ __forceinline__ uint64_t load_chunk_agents(const Params &p, int64_t c, uint64_t mask, bool multi,
                                                       int64_t &home, int &f)
{
    const int lane = lane_id();
    const int64_t pos = c * kWave + lane;
    bool agent = false;
    home = 0;
    f = 0;
    if ((mask >> lane) & 1ull) {
        uint32_t first;
        if (STORE_FIRST) {
            first = p.set_minpos[p.ent[pos]];
            p.first_of[pos] = first;
        } else {
            first = p.first_of[pos];
        }
        agent = first == (uint32_t)pos;
        if (agent) {
            const int64_t id = p.ids[pos];
            uint64_t seed = p.t0.seed;
            int64_t n_slots = p.t0.N;
            if (multi) {
                f = find_table(p.offsets, p.num_tables, pos);
                seed = p.descs[f].seed;
                n_slots = p.descs[f].N;
            }
            home = home_slot(id, seed, n_slots);
        }
    }
    return __ballot(agent);
}

// Hands the next (64 / G) set bits of amask to the groups of the wavefront: returns this
// group's bit index or -1, and removes the bits that were handed out.
template <int G>
__device__ __forceinline__ int next_agent(uint64_t &amask, int g)
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

// One G-lane group per elected position runs deferred acceptance for it: propose to the first
// slot of the window that is claimable and not held by a better tag; on displacing another tag
// continue on behalf of its owner.
template <int G>
__global__ __launch_bounds__(kBlock) void k_allocate(Params p)
{
    const int lane = lane_id();
    const int g = lane / G, r = lane % G;
    int64_t c_begin, c_end, wave_global;
    wave_chunk_range(p.n, c_begin, c_end, wave_global);
    const bool multi = p.num_tables > 1;

    for (int64_t c = c_begin; c < c_end; ++c) {
        const uint64_t mask = uniform64(p.miss_mask[c]);
        if (mask == 0) continue;
        int64_t lane_home;
        int lane_f;
        uint64_t amask = load_chunk_agents<true>(p, c, mask, multi, lane_home, lane_f);
        while (amask) {
            const int b = next_agent<G>(amask, g);
            // group-uniform state of the claimant carried by this group
            bool active = b >= 0;
            const int src = active ? b : 0;
            uint32_t cpos = (uint32_t)(c * kWave + src);   // its position (priority within a round)
            int64_t home = shfl64(lane_home, src);
            int32_t cr = 0;                                 // next round to try
            TableDesc d = p.t0;
            if (multi) d = p.descs[__shfl(lane_f, src)];
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
                            cmask &= ~(1ull << (g * G + first));
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
                            // carry the displaced claimant on from its next round (same table:
                            // both claimed the same slot)
                            cpos = tag_pos(displaced);
                            cr = (int32_t)tag_round(displaced) + 1;
                            home = home_slot(p.ids[cpos], d.seed, d.N);
                            if (cr >= d.P) active = false;   // out of rounds: falls back at finalize
                        } else {
                            active = false;
                        }
                    } else {
                        cr += G;
                        if (cr >= d.P) active = false;       // window exhausted: falls back at finalize
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------ finalize
// Appends the staged evicted slots of one wavefront to table `table`'s list.
__device__ __forceinline__ void flush_evicted(const Params &p, const int64_t *buf, int &count, int table)
{
    if (count == 0) return;
    const int lane = lane_id();
    unsigned long long base = 0;
    if (lane == 0) base = atomicAdd(&p.ctl->num_evicted[table], (unsigned long long)count);
    base = (unsigned long long)shfl64((int64_t)base, 0);
    const int64_t ev_begin = p.num_tables > 1 ? p.descs[table].ev_begin : p.t0.ev_begin;
    const int64_t ev_cap = p.num_tables > 1 ? p.descs[table].ev_cap : p.t0.ev_cap;
    for (int i = lane; i < count; i += kWave) {
        const int64_t at = (int64_t)base + i;
        if (at < ev_cap) p.out_evicted[ev_begin + at] = buf[i];
    }
    count = 0;
}

template <int G>
__global__ __launch_bounds__(kBlock) void k_finalize(Params p)
{
    __shared__ int64_t s_ev[kWavesPerBlock][kEvBuf];
    __shared__ int s_cnt[kWavesPerBlock];
    __shared__ int s_tab[kWavesPerBlock];
    __shared__ unsigned long long s_base;

    const int lane = lane_id();
    const int w = threadIdx.x / kWave;
    const int g = lane / G, r = lane % G;
    int64_t c_begin, c_end, wave_global;
    wave_chunk_range(p.n, c_begin, c_end, wave_global);
    const bool multi = p.num_tables > 1;
    const bool want_stats = p.out_stats != nullptr;

    int ev_cnt = 0, ev_table = 0;                       // wave-uniform
    unsigned long long st_ins = 0, st_evi = 0, st_col = 0;
    int st_table = 0;

    for (int64_t c = c_begin; c < c_end; ++c) {
        const uint64_t mask = uniform64(p.miss_mask[c]);
        if (mask == 0) continue;
        int64_t lane_home;
        int lane_f;
        uint64_t amask = load_chunk_agents<false>(p, c, mask, multi, lane_home, lane_f);
        while (amask) {
            const int b = next_agent<G>(amask, g);
            const bool active = b >= 0;
            const int src = active ? b : 0;
            const uint32_t cpos = (uint32_t)(c * kWave + src);
            const int64_t home = shfl64(lane_home, src);
            const int f = multi ? __shfl(lane_f, src) : 0;
            TableDesc d = p.t0;
            if (multi) d = p.descs[f];
            // counters are kept in registers for one table at a time; where a chunk straddles a
            // feature boundary (rare) they go straight to the per-table counters
            bool direct = false;
            if (want_stats && multi) {
                const uint64_t am = __ballot(active);
                const int f0 = __shfl(f, am ? __ffsll((unsigned long long)am) - 1 : 0);
                direct = __any(active && f != f0);
                if (f0 != st_table) {
                    if (st_ins) atomicAdd(&p.ctl->stats[st_table][kInserts], st_ins);
                    if (st_evi) atomicAdd(&p.ctl->stats[st_table][kEvictions], st_evi);
                    if (st_col) atomicAdd(&p.ctl->stats[st_table][kCollisions], st_col);
                    st_ins = st_evi = st_col = 0;
                    st_table = f0;
                }
            }
            // find the slot that carries this claimant's tag
            bool searching = active;
            bool found = false;
            bool ev_lane = false;        // this lane turned a tag on an occupied slot into the id
            int64_t ev_slot = 0;
            for (int32_t cc = 0; __any(searching); cc += G) {
                const int32_t round = cc + r;
                bool m = false;
                if (searching && round < d.P) {
                    const int64_t s = wrap(home + round, d.N);
                    const int64_t v = __hip_atomic_load(&d.I[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    m = is_tag(v) && tag_pos(v) == cpos;
                    if (m) {
                        // the claim becomes the id; metadata gets the step (Algorithm 1, Pass 2)
                        __hip_atomic_store(&d.I[s], p.ids[cpos], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        d.M[s] = p.step;
                        p.out_slots[cpos] = s;
                        if (tag_occ(v)) {
                            ev_lane = true;
                            ev_slot = s;
                            if (direct) atomicAdd(&p.ctl->stats[f][kEvictions], 1ull); else st_evi++;
                        } else {
                            if (direct) atomicAdd(&p.ctl->stats[f][kInserts], 1ull); else st_ins++;
                        }
                    }
                }
                const int first = group_first<G>(__ballot(m), g);
                if (searching) {
                    if (first >= 0) { found = true; searching = false; }
                    else if (cc + G >= d.P) searching = false;
                }
            }
            if (active && !found && r == 0) {
                // Case 3: no empty or evictable slot -> home slot, its metadata refreshed
                d.M[home] = p.step;
                p.out_slots[cpos] = home;
                if (direct) atomicAdd(&p.ctl->stats[f][kCollisions], 1ull); else st_col++;
            }
            // stage evicted slots in LDS; all entries of the buffer belong to one table
            uint64_t evm = __ballot(ev_lane);
            while (evm) {
                const int lead = __ffsll((unsigned long long)evm) - 1;
                const int tf = __shfl(f, lead);
                const bool sel = ev_lane && f == tf;
                const uint64_t selm = __ballot(sel);
                const int add = __popcll(selm);
                if ((ev_cnt > 0 && tf != ev_table) || ev_cnt + add > kEvBuf) {
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    flush_evicted(p, s_ev[w], ev_cnt, ev_table);
                }
                ev_table = tf;
                if (sel) s_ev[w][ev_cnt + __popcll(selm & ((1ull << lane) - 1ull))] = ev_slot;
                ev_cnt += add;
                evm &= ~selm;
            }
        }
    }

    // one reservation per workgroup when all its wavefronts staged for the same table
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (lane == 0) { s_cnt[w] = ev_cnt; s_tab[w] = ev_table; }
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
    if (total > 0) {
        if (same) {
            if (threadIdx.x == 0) s_base = atomicAdd(&p.ctl->num_evicted[tab], (unsigned long long)total);
            __syncthreads();
            const int64_t base = (int64_t)s_base + before;
            const int64_t ev_begin = multi ? p.descs[tab].ev_begin : p.t0.ev_begin;
            const int64_t ev_cap = multi ? p.descs[tab].ev_cap : p.t0.ev_cap;
            for (int i = lane; i < ev_cnt; i += kWave)
                if (base + i < ev_cap) p.out_evicted[ev_begin + base + i] = s_ev[w][i];
        } else {
            flush_evicted(p, s_ev[w], ev_cnt, ev_table);
        }
    }

    if (want_stats) {
        const unsigned long long a = wave_sum(st_ins), b2 = wave_sum(st_evi), x = wave_sum(st_col);
        if (lane == 0 && wave_global < p.waves_b) {
            StatRow row;
            for (int k = 0; k < kStatCount; ++k) row.v[k] = 0;
            row.v[kInserts] = a;
            row.v[kEvictions] = b2;
            row.v[kCollisions] = x;
            row.table = st_table;
            p.rows_b[wave_global] = row;
        }
    }
}

// ------------------------------------------------------------------ duplicates, cleanup, counters
__global__ __launch_bounds__(kBlock) void k_emit_dups(Params p)
{
    __shared__ unsigned long long s_bins[kMaxTables][kStatCount];
    const int lane = lane_id();
    int64_t c_begin, c_end, wave_global;
    wave_chunk_range(p.n, c_begin, c_end, wave_global);

    for (int64_t c = c_begin; c < c_end; ++c) {
        const uint64_t mask = uniform64(p.miss_mask[c]);
        if (!((mask >> lane) & 1ull)) continue;
        const int64_t pos = c * kWave + lane;
        const uint32_t first = p.first_of[pos];
        const uint32_t e = p.ent[pos];
        if (first != (uint32_t)pos) p.out_slots[pos] = p.out_slots[first];
        // empty the scratch set entry again (every copy of the id does; the stores agree)
        p.set_keys[e] = -1;
        p.set_minpos[e] = 0xFFFFFFFFu;
    }

    if (blockIdx.x == 0) {
        for (int i = threadIdx.x; i < p.num_tables; i += kBlock)
            p.out_num_evicted[i] = (int64_t)p.ctl->num_evicted[i];
        if (p.out_stats) {
            const int nbins = p.num_tables * kStatCount;
            for (int i = threadIdx.x; i < nbins; i += kBlock)
                s_bins[i / kStatCount][i % kStatCount] = p.ctl->stats[i / kStatCount][i % kStatCount];
            __syncthreads();
            for (int i = threadIdx.x; i < p.waves_a + p.waves_b; i += kBlock) {
                const StatRow *row = i < p.waves_a ? &p.rows_a[i] : &p.rows_b[i - p.waves_a];
                const int t = (int)row->table;
                for (int k = 0; k < kStatCount; ++k) {
                    const unsigned long long v = row->v[k];
                    if (v) atomicAdd(&s_bins[t][k], v);
                }
            }
            __syncthreads();
            for (int t = threadIdx.x; t < p.num_tables; t += kBlock)
                s_bins[t][kDistinctMiss] = s_bins[t][kInserts] + s_bins[t][kEvictions] + s_bins[t][kCollisions];
            __syncthreads();
            for (int i = threadIdx.x; i < nbins; i += kBlock)
                p.out_stats[i] = (int64_t)s_bins[i / kStatCount][i % kStatCount];
        }
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
