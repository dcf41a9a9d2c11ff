/*
 * mpzch.h -- C ABI of the MI355X (gfx950) batched MPZCH remap library.
 *
 * MPZCH ("Multi-Probe Zero Collision Hash") maps raw int64 feature ids to
 * embedding-table slots: hash to a home slot, probe at most max_probe
 * consecutive slots of an `identities` tensor, then hit / insert into an empty
 * slot / evict an expired id / fall back to the home slot (paper Sec. 3.2 and
 * Algorithm 1), with TTL eviction guided by a `metadata` tensor (Sec. 3.4) and
 * reset of the embedding rows of reassigned slots (Sec. 3.4, last paragraph).
 *
 * Conventions that hold for every call
 *   - DEVICE pointers are marked [dev], HOST pointers [host].  The caller owns
 *     every tensor (identities, metadata, ids, outputs, embedding rows); a handle
 *     owns only its configuration and a scratch area in device memory.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No call synchronises with the host unless stated.
 *   - One call per handle may be in flight at a time; calls issued on one stream
 *     are ordered.  Two calls that touch the same identities tensor must not
 *     overlap.
 *   - Errors come back as status codes; nothing aborts or throws.  Argument
 *     errors are found before anything is launched.  Data-dependent conditions
 *     (negative ids, a truncated evicted list) are reported through device-side
 *     counters, never through a host synchronisation.
 *
 * Definitions shared by all entry points (the paper leaves them open)
 *   hash(id)   = SplitMix64 finaliser of ((uint64)id XOR hash_seed)
 *   home(id)   = floor(hash(id) * num_slots / 2^64)
 *   slot(id,r) = (home(id) + r) mod num_slots,  0 <= r < min(max_probe, num_slots)
 *   empty slot : identities == -1            (Sec. 3.1)
 *   metadata   : step at which the slot's id was last seen (int32)
 *   expired    : policy TTL and  step - metadata > ttl     (Sec. 3.4)
 *   valid ids  : 0 <= id <= 2^63 - 1.  Negative ids are never stored and never
 *                match; their output is home(id) of their bit pattern.
 * Precondition on identities: it was initialised by mpzch_init_tensors and since then written
 * only by this library (or is a copy of such a tensor).  Such a table never has an empty slot
 * between an id's home and the slot that holds it -- an occupied slot never becomes empty again --
 * and the lookups use that: a search ends at the first empty slot of the probe range.
 * While mpzch_remap / mpzch_remap_jagged run, identities may transiently hold
 * values <= -2; they are gone when the call's work on the stream has finished.
 */
#ifndef MPZCH_H
#define MPZCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mpzch_table mpzch_table_t; /* opaque: configuration + device scratch   */
typedef struct mpzch_group mpzch_group_t; /* opaque: several tables remapped together */

typedef enum {
    MPZCH_OK = 0,
    MPZCH_ERR_INVALID_ARG = 1,
    MPZCH_ERR_ALLOC = 2,       /* device or host allocation failed */
    MPZCH_ERR_HIP = 3,         /* a HIP runtime call failed; when a remap returns it, the tensors may be
                                  left mid-update (their state is undefined), the handle stays usable */
    MPZCH_ERR_UNSUPPORTED = 4, /* e.g. MPZCH_EVICT_LRU with max_probe > MPZCH_MAX_PROBE_LRU */
    MPZCH_ERR_TOO_LARGE = 5    /* a size beyond the fixed maximum of an entry point that allocates nothing */
} mpzch_status_t;

typedef enum {
    MPZCH_EVICT_NONE = 0, /* lookup + insert only (Sec. 3.3, eviction disabled)           */
    MPZCH_EVICT_TTL = 1,  /* lazy TTL eviction (Sec. 3.4)                                 */
    MPZCH_EVICT_LRU = 2   /* Sec. 3.4 last paragraph: first empty slot of the range, else evict the entry
                             with the oldest metadata (ties: earlier probe round), never one whose metadata
                             equals the current step; contended slots go to the lower choice number, then
                             to the id whose first occurrence comes first.
                             max_probe <= MPZCH_MAX_PROBE_LRU only (else MPZCH_ERR_UNSUPPORTED). */
    , MPZCH_EVICT_TTL_EXPIRY = 3 /* Sec. 3.4 as written, for tables shared by features with different
                             retention ("per-feature TTL"): metadata holds the step after which the id is
                             expired, step + ttl of its feature; a slot is expired when metadata < step.
                             With one ttl for all ids this is MPZCH_EVICT_TTL with metadata shifted by ttl. */
} mpzch_evict_kind_t;

typedef struct {
    int32_t kind; /* mpzch_evict_kind_t         */
    int32_t ttl;  /* steps, >= 0; used with TTL */
} mpzch_eviction_policy_t;

/* Index of each counter in the int64 stats array written by the remap calls. */
enum {
    MPZCH_STAT_HIT_POS = 0,       /* positions whose id was resident at batch start        */
    MPZCH_STAT_MISS_POS = 1,      /* valid positions whose id was not resident             */
    MPZCH_STAT_DISTINCT_MISS = 2, /* distinct ids among the miss positions                 */
    MPZCH_STAT_INSERTS = 3,       /* distinct missed ids placed in an empty slot           */
    MPZCH_STAT_EVICTIONS = 4,     /* distinct missed ids placed by evicting an expired id  */
    MPZCH_STAT_COLLISIONS = 5,    /* distinct missed ids left without a slot (Table 1)     */
    MPZCH_STAT_INVALID_POS = 6,   /* positions holding a negative id                       */
    MPZCH_STAT_HIT_PROBE_SUM = 7, /* sum over hit positions of (probe distance + 1)        */
    MPZCH_STAT_MISS_PROBE_SUM = 8, /* sum over miss positions of the slots Pass 1 has to read: up to and
                                     including the first empty slot of the range, else the whole range */
    MPZCH_STAT_COUNT = 9
};

#define MPZCH_MAX_BATCH ((int64_t)1 << 30) /* positions per remap / lookup call          */
#define MPZCH_MAX_PROBE (1 << 20)          /* upper bound accepted for max_probe          */
#define MPZCH_MAX_SLOTS ((int64_t)1 << 40) /* upper bound accepted for num_slots (8 TB of identities) */
/* The identities of a table must lie below address 2^48 (every device address of this GPU does): the
   kernels keep the address of a slot in 48 bits.  Entry points that probe a table return INVALID_ARG
   for one that does not. */
#define MPZCH_MAX_GROUP_TABLES 64          /* tables per mpzch_group_t                    */
#define MPZCH_MAX_PROBE_LRU 1024           /* largest max_probe with MPZCH_EVICT_LRU      */

/*
 * Creates a table handle (Algorithm 1's globals: P = max_probe; Sec. 3.4: policy).
 * Allocates no tensor and touches no GPU: scratch is allocated by the first remap
 * (or by mpzch_reserve) on the device that is current then.
 * Errors: INVALID_ARG for num_slots < 1 or > MPZCH_MAX_SLOTS, max_probe < 1 or > MPZCH_MAX_PROBE, ttl < 0,
 * unknown policy kind, out == NULL; UNSUPPORTED for MPZCH_EVICT_LRU with max_probe > MPZCH_MAX_PROBE_LRU.
 * max_probe > num_slots is accepted and behaves as max_probe == num_slots.
 */
mpzch_status_t mpzch_create(int64_t num_slots, int32_t max_probe, mpzch_eviction_policy_t policy,
                            uint64_t hash_seed, mpzch_table_t **out /* [host] */);

/*
 * mpzch_create with a choice of where the two auxiliary tensors of Sec. 3.1 live:
 *   MPZCH_LAYOUT_SEPARATE  identities int64[num_slots] and metadata int32[num_slots], two dense tensors
 *                          (what mpzch_create gives);
 *   MPZCH_LAYOUT_RECORDS   ONE tensor of num_slots 16-byte records {int64 id; int32 metadata; int32 unused},
 *                          16-byte aligned.  Every entry point that takes `identities` / `metadata` for such a
 *                          table is given  identities = &record[0].id  and  metadata = &record[0].metadata
 *                          (= (int32_t *)identities + 2; anything else is INVALID_ARG); slot s is then the
 *                          int64 at identities + 2 s and the int32 at metadata + 4 s.  Same results slot by
 *                          slot.  The 128-byte line that a probe fetches holds the metadata word that a hit
 *                          refreshes, which saves the memory system one of the three random accesses a hit
 *                          costs on MI355X, for 16 instead of 12 bytes per slot.
 * mpzch_apply_delta writes dense identities only (the published copy of Sec. 3.7 carries no metadata).
 * INVALID_ARG for an unknown layout.
 */
typedef enum { MPZCH_LAYOUT_SEPARATE = 0, MPZCH_LAYOUT_RECORDS = 1 } mpzch_layout_t;
mpzch_status_t mpzch_create_with_layout(int64_t num_slots, int32_t max_probe, mpzch_eviction_policy_t policy,
                                        uint64_t hash_seed, int32_t layout, mpzch_table_t **out /* [host] */);

/* Frees the handle and its scratch.  Synchronises the device first.  NULL is accepted. */
mpzch_status_t mpzch_destroy(mpzch_table_t *t);

/*
 * Optional: allocate scratch for batches of up to max_n positions now (about 29 bytes per
 * position) so that later remap calls allocate nothing.  Synchronises the device when it
 * has to grow the scratch.  Errors: INVALID_ARG (max_n < 0 or > MPZCH_MAX_BATCH), ALLOC.
 * With enough scratch reserved and kernel timing off, mpzch_remap, mpzch_remap_feature_ttl,
 * mpzch_lookup and the row movers only launch kernels on the given stream (no allocation, no
 * synchronisation, no memset) and leave their counters zeroed for the next call, so a step may
 * be captured into a HIP graph and replayed (step and pointers are then those of the capture).
 */
mpzch_status_t mpzch_reserve(mpzch_table_t *t, int64_t max_n);

/*
 * Sec. 3.1 initial state: identities[0..num_slots) = -1, metadata[0..num_slots) = -1.
 * metadata may be NULL.  identities [dev] int64[num_slots], metadata [dev] int32[num_slots].
 */
mpzch_status_t mpzch_init_tensors(const mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                                  void *stream);

/*
 * Training remap of one batch: lookup, insert and evict (Sec. 3.2, Algorithm 1; Sec. 3.3
 * "Kernel Execution"; Sec. 3.4; Sec. 3.6 input de-duplication).  The batch is processed as
 *   1. every id resident at the start of the call is found (Pass 1) and its metadata set
 *      to `step` ("Update"), before anything is allocated;
 *   2. the remaining distinct ids allocate: each takes the first slot of its probe range
 *      that is empty or expired; where several ids want one slot the one that reaches it
 *      in the earlier probe round wins, and within a round the id whose first occurrence
 *      in the batch comes first; a claimed slot gets identities = id, metadata = step;
 *   3. ids left without a slot fall back to their home slot, whose metadata is set to
 *      `step` (Case 3);
 *   4. every position receives the slot of its id (all copies of an id share one slot).
 *
 * identities [dev] int64[num_slots]  in/out
 * metadata   [dev] int32[num_slots]  in/out
 * ids        [dev] int64[n]          raw ids, 0 <= n <= MPZCH_MAX_BATCH
 * step                               current time stamp, >= 0, non-decreasing over calls
 * out_slots  [dev] int64[n]          remapped index of every position
 * out_evicted_slots [dev] int64[evicted_cap]  slots that changed owner (Sec. 3.4: the rows
 *                                    to reset), each once, order unspecified; may be NULL
 *                                    when evicted_cap == 0
 * out_num_evicted   [dev] int64[1]   number of such slots; when it exceeds evicted_cap
 *                                    the list holds the first evicted_cap that were written
 * out_stats  [dev] int64[MPZCH_STAT_COUNT] or NULL
 * n == 0 is valid: outputs counts are written as zero, state is untouched.
 * Errors: INVALID_ARG (NULL handle / required pointer, n out of range, step < 0,
 * evicted_cap < 0), ALLOC (scratch), HIP.
 */
mpzch_status_t mpzch_remap(mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                           const int64_t *ids, int64_t n, int32_t step,
                           int64_t *out_slots,
                           int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                           int64_t *out_stats, void *stream);

/*
 * mpzch_remap that also resets the embedding rows of the slots it evicts (Sec. 3.4: the weights
 * of an evicted id must not be inherited by the id that takes its slot), in the kernel that
 * decides the evictions: rows[(slot mod num_rows), 0..row_bytes) <- init_row, or zero bits when
 * init_row is NULL, for EVERY slot that changed owner in this call -- also for those beyond
 * evicted_cap, which mpzch_remap + mpzch_reset_rows would leave out.  Otherwise identical to
 * mpzch_remap followed by mpzch_reset_rows (the evicted list and its count are still written, for
 * further tensors to reset with mpzch_reset_rows_multi); one launch less, and the list does not
 * travel through HBM before the rows are written.
 * rows [dev], num_rows >= 1, row_bytes, row_stride_bytes, init_row [dev]: as for mpzch_reset_rows.
 * Errors: those of mpzch_remap and of mpzch_reset_rows; INVALID_ARG when rows == NULL.
 */
mpzch_status_t mpzch_remap_reset(mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                                 const int64_t *ids, int64_t n, int32_t step,
                                 int64_t *out_slots,
                                 int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                                 int64_t *out_stats,
                                 void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                 const void *init_row, void *stream);

/*
 * mpzch_remap for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result and same kernels as
 * mpzch_remap, but the scratch is a fixed area of MPZCH_NOALLOC_SCRATCH_BYTES bytes that the library
 * holds in every GPU's memory from load until the process ends, instead of the handle's own; the handle
 * supplies the configuration only and is not modified.  The call allocates and frees nothing and never
 * synchronises.  The first call on a GPU also looks up that GPU's copy of the area and clears it
 * with two fill kernels on `stream`: make that call outside graph capture.
 * n > MPZCH_NOALLOC_MAX_BATCH is rejected with MPZCH_ERR_TOO_LARGE before anything is launched.
 * All calls on one GPU -- whatever the handle, whatever the stream -- share that GPU's area: calls that
 * overlap in time on one GPU race; order them on one stream or with events.  Every call leaves the
 * area ready for the next one (set emptied, counters zeroed).
 */
#define MPZCH_NOALLOC_MAX_BATCH ((int64_t)262144)
#define MPZCH_NOALLOC_SCRATCH_BYTES (9u << 20) /* 9 MiB per GPU */
mpzch_status_t mpzch_remap_noalloc(const mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                                   const int64_t *ids, int64_t n, int32_t step,
                                   int64_t *out_slots,
                                   int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                                   int64_t *out_stats, void *stream);

/*
 * mpzch_remap for a table of kind MPZCH_EVICT_TTL_EXPIRY whose ids come from features with different
 * retention (Sec. 3.4, second paragraph).  ttls [dev] int32[n]: retention in steps (>= 0) of the feature
 * each position belongs to; NULL = policy.ttl for all (then any table kind is accepted and the call is
 * mpzch_remap).  step + ttl must fit int32.
 * Metadata rule of this kind: a slot that is claimed gets metadata = step + ttl of the claiming id's
 * first occurrence; every other write is a refresh on behalf of one position -- a copy of the id that
 * lives in the slot (copies may carry different ttls), or an id that falls back to the slot as its home
 * (Case 3) -- and a refresh stores max(metadata, step + ttl of that position): the expiry step of a slot
 * never moves backward, so a short-lived feature cannot cut short the retention a long-lived one gave,
 * and the result does not depend on the order of the positions.  (Algorithm 1 as printed stores the
 * value of whichever position is processed last.)
 */
mpzch_status_t mpzch_remap_feature_ttl(mpzch_table_t *t, int64_t *identities, int32_t *metadata,
                                       const int64_t *ids, const int32_t *ttls, int64_t n, int32_t step,
                                       int64_t *out_slots,
                                       int64_t *out_evicted_slots, int64_t evicted_cap, int64_t *out_num_evicted,
                                       int64_t *out_stats, void *stream);

/*
 * Inference lookup (Sec. 3.7): read-only, Pass 1 of Algorithm 1 for every position
 * independently; needs no metadata and no scratch.
 * out_slots [dev] int64[n]: the slot holding the id, or home(id) when it is not resident.
 * out_found [dev] uint8[n] or NULL: 1 when resident.
 */
mpzch_status_t mpzch_lookup(const mpzch_table_t *t, const int64_t *identities,
                            const int64_t *ids, int64_t n,
                            int64_t *out_slots, uint8_t *out_found, void *stream);

/*
 * mpzch_lookup that also counts (Sec. 3.7; the numbers a serving system watches, and what the benchmark's
 * byte accounting needs): out_stats [dev] int64[MPZCH_STAT_COUNT] receives HIT_POS, MISS_POS, INVALID_POS,
 * HIT_PROBE_SUM and MISS_PROBE_SUM of this call (the other entries are written as zero).  Uses a small
 * counter block owned by the handle (allocated by the first such call, which synchronises the device
 * once), hence the non-const handle; one counting lookup or remap per handle at a time.
 */
mpzch_status_t mpzch_lookup_stats(mpzch_table_t *t, const int64_t *identities,
                                  const int64_t *ids, int64_t n,
                                  int64_t *out_slots, uint8_t *out_found, int64_t *out_stats, void *stream);

/*
 * Reset of reassigned rows (Sec. 3.4: "upon eviction, both the embedding weights and the
 * optimizer state are reset"): for k < min(*num_slots_dev, slots_cap):
 *     rows[(slots[k] mod num_rows) * row_stride_bytes .. + row_bytes) <- init_row
 * slots         [dev] int64[slots_cap]   e.g. out_evicted_slots of mpzch_remap
 * num_slots_dev [dev] int64[1]           e.g. out_num_evicted; read on the device, so no
 *                                        host synchronisation sits between remap and reset
 * rows          [dev] any dtype; row_bytes > 0 and row_stride_bytes >= row_bytes, both
 *               multiples of 4; rows 4-byte aligned (16-byte alignment of rows, stride and
 *               row_bytes enables 128-bit stores)
 * init_row      [dev] row_bytes bytes, or NULL for all-zero bits
 * Call it once per tensor that has to be reset (weights, optimizer state).
 */
mpzch_status_t mpzch_reset_rows(const int64_t *slots, const int64_t *num_slots_dev, int64_t slots_cap,
                                void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                const void *init_row, void *stream);

/*
 * Reset of several tensors in one launch (Sec. 3.4: "both the embedding weights and the optimizer
 * state (e.g., momentum) are reset"): as mpzch_reset_rows for each of tensors[0 .. num_tensors).
 * tensors [host] array of 1..4 descriptions; every field as in mpzch_reset_rows.
 */
typedef struct {
    void *rows;               /* [dev] */
    int64_t num_rows;
    int64_t row_bytes;
    int64_t row_stride_bytes;
    const void *init_row;     /* [dev] row_bytes bytes, or NULL for zeros */
} mpzch_rows_t;
mpzch_status_t mpzch_reset_rows_multi(const int64_t *slots, const int64_t *num_slots_dev, int64_t slots_cap,
                                      const mpzch_rows_t *tensors, int32_t num_tensors, void *stream);

/*
 * Inference lookup fused with the embedding gather (Sec. 3.7), one kernel: the lanes that resolve the
 * slots of 64 ids copy their rows, out_rows[j, :] = rows[slot_j mod num_rows, :], where slot_j is what
 * mpzch_lookup returns for ids[j] (the home slot's row when the id is not resident).
 * rows as in mpzch_reset_rows; out_rows [dev] n x row_bytes bytes, dense; row_bytes <= 16 MiB.
 * out_slots [dev] int64[n] or NULL: the looked-up slots, written only when given.
 * out_found [dev] uint8[n] or NULL.
 */
mpzch_status_t mpzch_lookup_gather(const mpzch_table_t *t, const int64_t *identities,
                                   const int64_t *ids, int64_t n,
                                   const void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                   void *out_rows, int64_t *out_slots, uint8_t *out_found, void *stream);

/*
 * Streaming delta (Sec. 3.8: sparse delta publishing; "the corresponding entries in the identities tensor
 * are updated in conjunction with the embedding rows").
 *
 * mpzch_collect_delta (training side): every occupied slot whose metadata is >= since_step -- the slots
 * whose id was seen, inserted or refreshed since then -- goes to the list (out_slots[k], out_ids[k]), order
 * unspecified.  out_count [dev] int64[1] receives the number found; when it exceeds cap the lists hold the
 * first cap that were written.  Needs metadata that holds last-seen steps (TTL, LRU or no eviction).
 *
 * mpzch_gather_rows: out_rows[k, :] = rows[slots[k] mod num_rows, :] for k < min(*count_dev, cap)
 * (count_dev may be NULL: then cap rows) -- the payload of a delta.
 *
 * mpzch_apply_delta (inference side): for k < min(*count_dev, cap): first
 * rows[slots[k] mod num_rows, :] = delta_rows[k, :], then identities[slots[k]] = ids[k].  rows may be NULL
 * (identities only).  Slots outside [0, num_slots) are skipped.
 */
mpzch_status_t mpzch_collect_delta(const mpzch_table_t *t, const int64_t *identities, const int32_t *metadata,
                                   int32_t since_step, int64_t *out_slots, int64_t *out_ids, int64_t cap,
                                   int64_t *out_count, void *stream);
mpzch_status_t mpzch_gather_rows(const int64_t *slots, const int64_t *count_dev, int64_t cap,
                                 const void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                 void *out_rows, void *stream);
mpzch_status_t mpzch_apply_delta(int64_t *identities, int64_t num_slots,
                                 const int64_t *slots, const int64_t *ids, const int64_t *count_dev, int64_t cap,
                                 void *rows, int64_t num_rows, int64_t row_bytes, int64_t row_stride_bytes,
                                 const void *delta_rows, void *stream);

/*
 * Several tables remapped by one launch sequence (Sec. 3.4: one kernel serving tables of
 * several features; Sec. 3.6: a keyed jagged batch of an embedding collection).
 * tables [host] array of num_tables handles (1..MPZCH_MAX_GROUP_TABLES); the group keeps
 * copies of their configuration, the handles may be destroyed afterwards.
 */
mpzch_status_t mpzch_group_create(mpzch_table_t *const *tables, int32_t num_tables,
                                  mpzch_group_t **out /* [host] */);
mpzch_status_t mpzch_group_destroy(mpzch_group_t *g);
mpzch_status_t mpzch_group_reserve(mpzch_group_t *g, int64_t max_total_values);

/*
 * Feature-major keyed jagged batch: feature f owns values[feature_offsets[f] ..
 * feature_offsets[f+1]) and is remapped into table f exactly as mpzch_remap would remap
 * that slice on its own (positions compare by their order inside the slice).
 *
 * identities [host] array of num_tables [dev] int64 pointers (table f: num_slots_f entries)
 * metadata   [host] array of num_tables [dev] int32 pointers
 *            (the first call, and any call whose pointers differ from the previous one,
 *            synchronises `stream` once to upload them)
 * values     [dev] int64[total_values]
 * feature_offsets [dev] int64[num_tables + 1], non-decreasing, [0] == 0, [num_tables] == total_values
 * out_slots  [dev] int64[total_values]   slot inside the table of the value's feature
 * out_evicted_slots [dev] int64, table f's list starts at evicted_offsets[f] and has room for
 *            evicted_offsets[f+1] - evicted_offsets[f] entries
 * evicted_offsets   [host] int64[num_tables + 1], non-decreasing
 * out_num_evicted   [dev] int64[num_tables]
 * out_stats  [dev] int64[num_tables * MPZCH_STAT_COUNT] or NULL
 */
mpzch_status_t mpzch_remap_jagged(mpzch_group_t *g, int64_t *const *identities, int32_t *const *metadata,
                                  const int64_t *values, const int64_t *feature_offsets,
                                  int64_t total_values, int32_t step,
                                  int64_t *out_slots,
                                  int64_t *out_evicted_slots, const int64_t *evicted_offsets,
                                  int64_t *out_num_evicted, int64_t *out_stats, void *stream);

/*
 * mpzch_remap_jagged for groups with tables of kind MPZCH_EVICT_TTL_EXPIRY whose region of the
 * batch mixes features of different retention (Sec. 3.4, second paragraph: several features share
 * one table).  ttls [dev] int32[total_values]: retention in steps (>= 0) of the feature each value
 * belongs to, read for the values of MPZCH_EVICT_TTL_EXPIRY tables only (copies of an id may carry
 * different values: metadata rule of mpzch_remap_feature_ttl); NULL = every table's own policy.ttl.
 * INVALID_ARG when ttls is given and no table of the group has that kind.
 */
mpzch_status_t mpzch_remap_jagged_feature_ttl(mpzch_group_t *g, int64_t *const *identities, int32_t *const *metadata,
                                              const int64_t *values, const int32_t *ttls,
                                              const int64_t *feature_offsets,
                                              int64_t total_values, int32_t step,
                                              int64_t *out_slots,
                                              int64_t *out_evicted_slots, const int64_t *evicted_offsets,
                                              int64_t *out_num_evicted, int64_t *out_stats, void *stream);

/*
 * Row reset (Sec. 3.4) after mpzch_remap_jagged, for all tables of the group in one launch: for table f
 * and every k < min(num_evicted[f], evicted_offsets[f+1] - evicted_offsets[f]) the row
 * (evicted_slots[evicted_offsets[f] + k] mod tensors[f].num_rows) of tensors[f] receives tensors[f].init_row
 * (zeros when NULL), as mpzch_reset_rows does for one table.
 * evicted_slots, num_evicted [dev]: the outputs of mpzch_remap_jagged; evicted_offsets [host] int64[T + 1]: the
 * same array; tensors [host] array of T row tensors (rows == NULL: nothing to reset for that table).
 * A change of pointers synchronises `stream` once to upload them.
 */
mpzch_status_t mpzch_reset_rows_jagged(mpzch_group_t *g, const int64_t *evicted_slots, const int64_t *evicted_offsets,
                                       const int64_t *num_evicted, const mpzch_rows_t *tensors, void *stream);

/*
 * Inference lookup (Sec. 3.7) for a feature-major keyed jagged batch: value k of feature f is looked
 * up in table f exactly as mpzch_lookup would, in one launch for all tables.  Read-only.
 * identities [host] array of num_tables [dev] const int64 pointers (a change of pointers synchronises
 *            `stream` once to upload them); values, feature_offsets, out_slots as in mpzch_remap_jagged;
 * out_found [dev] uint8[total_values] or NULL.
 */
mpzch_status_t mpzch_lookup_jagged(mpzch_group_t *g, const int64_t *const *identities,
                                   const int64_t *values, const int64_t *feature_offsets, int64_t total_values,
                                   int64_t *out_slots, uint8_t *out_found, void *stream);

/*
 * Per-kernel timing for benchmarks.  enable = 1: every kernel launched through the handle is
 * bracketed by HIP events on the call's stream; enable = 2: only the Pass-1 kernel of each call
 * (k_discover / k_lookup), which costs the call some eight microseconds instead of thirty;
 * enable = 3: the Pass-1 kernel of every fourth call (the 4th, 8th, ... after this call: a
 * sample, two microseconds per call on average); enable = 0: off.  mpzch_kernel_times
 * synchronises those events, adds up the durations per kernel and clears the record.
 * names [host] receives up to cap pointers to static strings, ms [host] the summed
 * milliseconds, launches [host] the number of launches; *count the number of kernels.
 */
mpzch_status_t mpzch_set_kernel_timing(mpzch_table_t *t, int32_t enable);
mpzch_status_t mpzch_kernel_times(mpzch_table_t *t, const char **names, double *ms, int64_t *launches,
                                  int32_t cap, int32_t *count);
mpzch_status_t mpzch_group_set_kernel_timing(mpzch_group_t *g, int32_t enable);
mpzch_status_t mpzch_group_kernel_times(mpzch_group_t *g, const char **names, double *ms, int64_t *launches,
                                        int32_t cap, int32_t *count);

const char *mpzch_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* MPZCH_H */
