/*
 * MPZCH oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, sequential, single-threaded CPU statement of what the batched
 * remap path computes.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load this file; the product path (the HIP library)
 * shares no code with it and never calls it.
 *
 * What it follows (paper: "Multi-Probe Zero Collision Hash"):
 *   - Sec. 3.1 (Auxiliary Tensors): identities I (int64, empty = -1) and
 *     metadata M (here: int32 last-seen step).
 *   - Sec. 3.2 + Algorithm 1: hash to a home slot, Pass 1 (discovery, read
 *     only), Pass 2 (update / insert / evict), Case 3 (collision fallback to
 *     the home slot, metadata of the home slot refreshed).
 *   - Sec. 3.4 (Eviction Management): lazy TTL eviction -- a new ID takes
 *     the first expired slot in its probe range; evicted slots are reported
 *     so that the embedding rows can be reset.
 *   - Sec. 3.6: input de-duplication (every copy of an ID gets one slot).
 *   - Sec. 3.7: inference lookup is read-only.
 *
 * Readings where the paper is silent (the same readings bind the HIP path):
 *   hash        = SplitMix64 finaliser of (id XOR seed);
 *   home        = floor(hash * N / 2^64)          (multiply-high);
 *   probe r     = (home + r) mod N, r < min(P, N) (window wraps);
 *   expired     = step - M[s] > ttl               (M holds the last-seen step);
 *   batch rule  = hits are refreshed before any allocation; misses allocate
 *                 round-major / first-occurrence-position-minor, so that in
 *                 every probe round the lowest first-occurrence batch index
 *                 wins a contended slot;
 *   invalid ids = negative ids: never stored, never match, map to the home
 *                 slot of their bit pattern;
 *   LRU policy  = first empty slot of the range, else the entry with the oldest
 *                 time stamp (ties: earlier round), never one seen at this step;
 *                 contended slots go to the lower choice number, then to the
 *                 lower first-occurrence batch index.
 *
 * Pins (tests/test_oracle_*.py): published SplitMix64 vectors; Table 1 of
 * the paper at reduced scale; the balls-in-bins closed form for P = 1;
 * textbook linear probing for P = N; a literal single-ID Algorithm 1 for
 * batch size 1; exhaustive stable-matching enumeration for the batch rule;
 * hand-worked TTL scenarios.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_EVICT_NONE = 0, ORACLE_EVICT_TTL = 1, ORACLE_EVICT_LRU = 2, ORACLE_EVICT_TTL_EXPIRY = 3 };

typedef struct {
    int64_t  num_slots;   /* N */
    int32_t  max_probe;   /* P */
    int32_t  policy;      /* ORACLE_EVICT_* */
    int32_t  ttl;         /* steps */
    int32_t  pad_;
    uint64_t hash_seed;
} oracle_cfg;

/* stats layout shared by name (not by code) with the HIP library */
enum {
    ST_HIT_POS = 0,      /* positions whose id was resident at batch start   */
    ST_MISS_POS,         /* valid positions whose id was not resident        */
    ST_DISTINCT_MISS,    /* distinct ids among the miss positions            */
    ST_INSERTS,          /* distinct missed ids placed in an empty slot      */
    ST_EVICTIONS,        /* distinct missed ids placed by evicting           */
    ST_COLLISIONS,       /* distinct missed ids that fell back to home       */
    ST_INVALID_POS,      /* positions holding a negative id                  */
    ST_HIT_PROBE_SUM,    /* sum over hit positions of (probe distance + 1)   */
    ST_MISS_PROBE_SUM,   /* sum over miss positions of the slots Pass 1 has to read: up to and
                            including the first empty slot of the range, else the whole range */
    ST_COUNT
};

/* SplitMix64 output function (public domain, Steele/Lea/Flood). */
uint64_t oracle_mix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Algorithm 1, "h <- Hash(id)": uniform over [0, N). */
int64_t oracle_home(int64_t id, uint64_t seed, int64_t num_slots)
{
    uint64_t h = oracle_mix64((uint64_t)id ^ seed);
    return (int64_t)(((unsigned __int128)h * (unsigned __int128)(uint64_t)num_slots) >> 64);
}

static int64_t p_eff(const oracle_cfg *c)
{
    return c->max_probe < c->num_slots ? (int64_t)c->max_probe : c->num_slots;
}

static int64_t probe_slot(int64_t home, int64_t r, int64_t n_slots)
{
    return (home + r) % n_slots;
}

/* Sec. 3.4: an occupied slot is reclaimable once its last-seen step is more
 * than ttl steps old; Sec. 3.1: an empty slot (-1) is always available. */
static int claimable(const oracle_cfg *c, const int64_t *I, const int32_t *M,
                     int64_t s, int32_t step)
{
    if (I[s] == -1) return 1;
    if (c->policy == ORACLE_EVICT_TTL && I[s] >= 0 &&
        (int64_t)step - (int64_t)M[s] > (int64_t)c->ttl) return 1;
    /* Sec. 3.4 as written: the stored value is "now + duration" of the id's feature, and a slot
     * whose value lies before the current time stamp is expired */
    if (c->policy == ORACLE_EVICT_TTL_EXPIRY && I[s] >= 0 && M[s] < step) return 1;
    return 0;
}

/* Pass 1 of Algorithm 1: first r with I[slot(r)] == id, else -1. */
static int64_t discover(const oracle_cfg *c, const int64_t *I, int64_t id, int64_t home)
{
    int64_t P = p_eff(c);
    for (int64_t r = 0; r < P; ++r)
        if (I[probe_slot(home, r, c->num_slots)] == id) return r;
    return -1;
}

typedef struct { int64_t id; int64_t pos; } id_pos;

static int cmp_id_pos(const void *a, const void *b)
{
    const id_pos *x = (const id_pos *)a, *y = (const id_pos *)b;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

/*
 * One training batch: insert + evict.  Returns 0, or -1 on bad arguments /
 * out of memory.  out_evicted receives at most evicted_cap slots (in claim
 * order); *out_num_evicted is the true count.  stats may be NULL.
 */
/* value written to the metadata of a slot touched for the id at batch position j */
static int32_t meta_value(const oracle_cfg *c, const int32_t *ttls, int64_t j, int32_t step)
{
    if (c->policy != ORACLE_EVICT_TTL_EXPIRY) return step;          /* last-seen step */
    return step + (ttls ? ttls[j] : c->ttl);                        /* per-feature TTL: expiry time */
}

/* "Refresh TTL" (Algorithm 1) of slot s, which keeps its occupant, on behalf of one batch position.
 * Last-seen metadata: M[s] = step, as printed.  Expiry-step metadata (Sec. 3.4, second paragraph:
 * features of different retention share a table): the slot keeps the LATEST expiry step any
 * processing of its occupant has asked for -- a refresh never moves it backward -- so a position of
 * a short-lived feature cannot cut short the retention a long-lived feature gave the slot, and the
 * outcome does not depend on the order in which the positions of a batch are taken. */
static void refresh(const oracle_cfg *c, int32_t *M, int64_t s, int32_t value)
{
    if (c->policy != ORACLE_EVICT_TTL_EXPIRY || value > M[s]) M[s] = value;
}

/* ttls: with ORACLE_EVICT_TTL_EXPIRY, the retention (in steps) of the feature each position
 * belongs to (Sec. 3.4, per-feature TTL); NULL = the table's ttl for every position.  Copies of
 * an id may carry different values: every copy refreshes the id's slot (see refresh). */
int oracle_remap_ttls(const oracle_cfg *c, int64_t *I, int32_t *M,
                      const int64_t *ids, const int32_t *ttls, int64_t n, int32_t step,
                      int64_t *out_slots,
                      int64_t *out_evicted, int64_t evicted_cap, int64_t *out_num_evicted,
                      int64_t *stats)
{
    if (!c || c->num_slots < 1 || c->max_probe < 1 || n < 0) return -1;
    int64_t st[ST_COUNT];
    memset(st, 0, sizeof st);
    int64_t n_evicted = 0;
    const int64_t N = c->num_slots, P = p_eff(c);

    if (n > 0) {
        /* Stage 0 (Sec. 3.6 de-duplication): first occurrence of every id. */
        id_pos *sorted = (id_pos *)malloc((size_t)n * sizeof *sorted);
        int64_t *first = (int64_t *)malloc((size_t)n * sizeof *first);   /* first-occurrence position */
        int64_t *result = (int64_t *)malloc((size_t)n * sizeof *result); /* slot, valid at first positions */
        int64_t *miss = (int64_t *)malloc((size_t)n * sizeof *miss);     /* first positions of missed ids */
        if (!sorted || !first || !result || !miss) {
            free(sorted); free(first); free(result); free(miss);
            return -1;
        }
        for (int64_t j = 0; j < n; ++j) { sorted[j].id = ids[j]; sorted[j].pos = j; }
        qsort(sorted, (size_t)n, sizeof *sorted, cmp_id_pos);
        for (int64_t k = 0; k < n; ++k) {
            if (k > 0 && sorted[k].id == sorted[k - 1].id)
                first[sorted[k].pos] = first[sorted[k - 1].pos];
            else
                first[sorted[k].pos] = sorted[k].pos;
        }
        free(sorted);

        /* Stage 1 (Pass 1 + "Update"): residents are found and refreshed
         * before any allocation happens.  Only M is written, only I is read,
         * so every id is discovered against the batch-start identities. */
        int64_t n_miss = 0;
        for (int64_t j = 0; j < n; ++j) {
            if (first[j] != j) continue;
            int64_t id = ids[j];
            int64_t h = oracle_home(id, c->hash_seed, N);
            if (id < 0) { result[j] = h; continue; }           /* invalid: no state change */
            int64_t r = discover(c, I, id, h);
            if (r >= 0) {
                result[j] = probe_slot(h, r, N);
            } else {
                result[j] = -1;
                miss[n_miss++] = j;                             /* ascending position */
            }
        }
        /* "Update": every position of a resident id refreshes its slot; per-position hit
         * statistics (duplicates included) */
        for (int64_t j = 0; j < n; ++j) {
            int64_t f = first[j];
            if (ids[j] < 0) { st[ST_INVALID_POS]++; continue; }
            if (result[f] >= 0) {
                int64_t h = oracle_home(ids[j], c->hash_seed, N);
                refresh(c, M, result[f], meta_value(c, ttls, j, step));
                st[ST_HIT_POS]++;
                st[ST_HIT_PROBE_SUM] += ((result[f] - h + N) % N) + 1;
            } else {
                /* no id lies beyond an empty slot of its range (a slot never becomes empty again),
                 * so that is as far as a search for an absent id has to read */
                int64_t h = oracle_home(ids[j], c->hash_seed, N), len = P;
                for (int64_t r = 0; r < P; ++r)
                    if (I[probe_slot(h, r, N)] == -1) { len = r + 1; break; }
                st[ST_MISS_POS]++;
                st[ST_MISS_PROBE_SUM] += len;
            }
        }
        st[ST_DISTINCT_MISS] = n_miss;

        if (c->policy == ORACLE_EVICT_LRU) {
            /* Stage 2, LRU policy (Sec. 3.4, last paragraph): a missed id takes the first
             * empty slot of its range; if there is none it evicts the entry with the oldest
             * time stamp (ties: the earlier probe round).  Entries seen at this very step are
             * never evicted.  Every missed id therefore has a preference list -- empty slots
             * in probe order, then evictable slots oldest first -- fixed by the state after
             * Stage 1.  Choice-major, position-minor sweep: in sweep k every id still
             * without a slot asks for its k-th choice, lowest batch position first. */
            int32_t *pref = (int32_t *)malloc((size_t)(n_miss > 0 ? n_miss : 1) * (size_t)P * sizeof *pref);
            int32_t *plen = (int32_t *)malloc((size_t)(n_miss > 0 ? n_miss : 1) * sizeof *plen);
            if (!pref || !plen) { free(pref); free(plen); free(first); free(result); free(miss); return -1; }
            for (int64_t k = 0; k < n_miss; ++k) {
                int64_t h = oracle_home(ids[miss[k]], c->hash_seed, N);
                int32_t *pl = pref + k * P;
                int32_t len = 0;
                for (int64_t r = 0; r < P; ++r)
                    if (I[probe_slot(h, r, N)] == -1) pl[len++] = (int32_t)r;
                int32_t start = len;
                for (int64_t r = 0; r < P; ++r) {
                    int64_t s = probe_slot(h, r, N);
                    if (I[s] < 0 || M[s] == step) continue;
                    int32_t at = len;                    /* insertion keeps (M, round) ascending */
                    while (at > start && M[probe_slot(h, pl[at - 1], N)] > M[s]) { pl[at] = pl[at - 1]; --at; }
                    pl[at] = (int32_t)r;
                    ++len;
                }
                plen[k] = len;
            }
            for (int64_t choice = 0; choice < P; ++choice) {
                for (int64_t k = 0; k < n_miss; ++k) {
                    int64_t j = miss[k];
                    if (result[j] >= 0 || choice >= plen[k]) continue;
                    int64_t s = probe_slot(oracle_home(ids[j], c->hash_seed, N), pref[k * P + choice], N);
                    if (I[s] != -1 && M[s] == step) continue;        /* taken earlier in this batch */
                    int was_occupied = (I[s] != -1);
                    I[s] = ids[j];
                    M[s] = step;
                    result[j] = s;
                    if (was_occupied) {
                        if (out_evicted && n_evicted < evicted_cap) out_evicted[n_evicted] = s;
                        n_evicted++;
                        st[ST_EVICTIONS]++;
                    } else {
                        st[ST_INSERTS]++;
                    }
                }
            }
            free(pref); free(plen);
        }

        /* Stage 2 (Pass 2 "Allocation", outcomes 1 and 2), TTL policy or eviction off:
         * round-major, position-minor.  A claim writes M = step, so the slot is no longer
         * claimable for anyone visiting it later in this batch. */
        for (int64_t r = 0; r < P && c->policy != ORACLE_EVICT_LRU; ++r) {
            for (int64_t k = 0; k < n_miss; ++k) {
                int64_t j = miss[k];
                if (result[j] >= 0) continue;
                int64_t id = ids[j];
                int64_t s = probe_slot(oracle_home(id, c->hash_seed, N), r, N);
                if (!claimable(c, I, M, s, step)) continue;
                int was_occupied = (I[s] != -1);
                I[s] = id;
                M[s] = meta_value(c, ttls, j, step);
                result[j] = s;
                if (was_occupied) {
                    if (out_evicted && n_evicted < evicted_cap) out_evicted[n_evicted] = s;
                    n_evicted++;
                    st[ST_EVICTIONS]++;
                } else {
                    st[ST_INSERTS]++;
                }
            }
        }

        /* Stage 3 (Case 3, collision fallback): home slot, its metadata refreshed ("M[h] <- meta";
         * the home slot keeps its occupant, so this is a refresh in the sense above). */
        char *missed = (char *)calloc((size_t)n, 1);              /* first positions of missed ids */
        if (!missed) { free(first); free(result); free(miss); return -1; }
        for (int64_t k = 0; k < n_miss; ++k) {
            int64_t j = miss[k];
            missed[j] = 1;
            if (result[j] >= 0) continue;
            int64_t h = oracle_home(ids[j], c->hash_seed, N);
            result[j] = h;
            refresh(c, M, h, meta_value(c, ttls, j, step));
            st[ST_COLLISIONS]++;
        }

        /* Stage 4: every copy of an id receives the slot of its first occurrence; the later
         * copies of an id that was placed or fell back in this batch refresh that slot too
         * (with one value per id, or last-seen metadata, this changes nothing). */
        for (int64_t j = 0; j < n; ++j) {
            out_slots[j] = result[first[j]];
            if (first[j] != j && ids[j] >= 0 && missed[first[j]])
                refresh(c, M, out_slots[j], meta_value(c, ttls, j, step));
        }
        free(missed);

        free(first); free(result); free(miss);
    }
    if (out_num_evicted) *out_num_evicted = n_evicted;
    if (stats) memcpy(stats, st, sizeof st);
    return 0;
}

int oracle_remap(const oracle_cfg *c, int64_t *I, int32_t *M,
                 const int64_t *ids, int64_t n, int32_t step,
                 int64_t *out_slots,
                 int64_t *out_evicted, int64_t evicted_cap, int64_t *out_num_evicted,
                 int64_t *stats)
{
    return oracle_remap_ttls(c, I, M, ids, NULL, n, step, out_slots, out_evicted, evicted_cap,
                             out_num_evicted, stats);
}

/* Sec. 3.7: read-only lookup.  Miss -> home slot, found flag 0.  stats (may be NULL) receives the
 * per-position counters of the call: hit / miss / invalid positions and the two probe-length sums. */
int oracle_lookup(const oracle_cfg *c, const int64_t *I,
                  const int64_t *ids, int64_t n,
                  int64_t *out_slots, uint8_t *out_found, int64_t *stats)
{
    if (!c || c->num_slots < 1 || c->max_probe < 1 || n < 0) return -1;
    int64_t st[ST_COUNT];
    memset(st, 0, sizeof st);
    const int64_t N = c->num_slots, P = p_eff(c);
    for (int64_t j = 0; j < n; ++j) {
        int64_t id = ids[j];
        int64_t h = oracle_home(id, c->hash_seed, N);
        int64_t r = id >= 0 ? discover(c, I, id, h) : -1;
        out_slots[j] = r >= 0 ? probe_slot(h, r, N) : h;
        if (out_found) out_found[j] = (uint8_t)(r >= 0);
        if (id < 0) {
            st[ST_INVALID_POS]++;
        } else if (r >= 0) {
            st[ST_HIT_POS]++;
            st[ST_HIT_PROBE_SUM] += r + 1;
        } else {
            int64_t len = P;                   /* as far as a search for an absent id has to read */
            for (int64_t k = 0; k < P; ++k)
                if (I[probe_slot(h, k, N)] == -1) { len = k + 1; break; }
            st[ST_MISS_POS]++;
            st[ST_MISS_PROBE_SUM] += len;
        }
    }
    if (stats) memcpy(stats, st, sizeof st);
    return 0;
}

/* Sec. 3.4: rows of reassigned slots go back to their initial value.
 * row index = slot mod num_rows; init_row == NULL means all-zero bytes. */
int oracle_reset_rows(const int64_t *slots, int64_t count,
                      uint8_t *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                      const uint8_t *init_row)
{
    if (count < 0 || num_rows < 1 || row_bytes < 0 || row_stride_bytes < row_bytes) return -1;
    for (int64_t k = 0; k < count; ++k) {
        if (slots[k] < 0) return -1;
        uint8_t *dst = rows + (slots[k] % num_rows) * row_stride_bytes;
        if (init_row) memcpy(dst, init_row, (size_t)row_bytes);
        else memset(dst, 0, (size_t)row_bytes);
    }
    return 0;
}

/*
 * State checker over slots [lo, hi): every resident id must be found by a
 * read-only lookup at exactly the slot that holds it.  That single condition
 * implies that no id is stored twice and that every resident lies within
 * min(P, N) probes of its home.  It also checks that no empty slot lies between
 * a resident's home and its slot.  Also counts occupied slots and slots holding
 * values that are neither -1 nor a valid id.  Returns the number of
 * violations; *first_bad is the first offending slot (or -1).
 */
int64_t oracle_check_state(const oracle_cfg *c, const int64_t *I,
                           int64_t lo, int64_t hi,
                           int64_t *out_occupied, int64_t *first_bad)
{
    int64_t bad = 0, occ = 0, fb = -1;
    for (int64_t s = lo; s < hi; ++s) {
        int64_t x = I[s];
        if (x == -1) continue;
        if (x < -1) { if (fb < 0) fb = s; bad++; continue; }
        occ++;
        int64_t h = oracle_home(x, c->hash_seed, c->num_slots);
        int64_t r = discover(c, I, x, h);
        if (r < 0 || probe_slot(h, r, c->num_slots) != s) { if (fb < 0) fb = s; bad++; continue; }
        /* a slot never becomes empty again, so no empty slot may precede a resident in its window */
        for (int64_t k = 0; k < r; ++k)
            if (I[probe_slot(h, k, c->num_slots)] == -1) { if (fb < 0) fb = s; bad++; break; }
    }
    if (out_occupied) *out_occupied = occ;
    if (first_bad) *first_bad = fb;
    return bad;
}
