/*
 * bagpipe.h — C ABI of the MI355X (gfx950) embedding-access hot path for lookahead-cached
 * recommendation-model training (Bagpipe, arXiv 2202.12429).
 *
 * The four operations follow the paper's division of labour (Section 3.1 "Design Overview",
 * Section 3.4): the Oracle Cacher plans, the trainer maintains a cache in GPU memory against
 * embedding servers, and the trainer runs the embedding forward / backward on cached rows.
 *
 *   bp_oracle_plan        lookahead planner (Algorithm 1 "Lookahead Algorithm", Section 3.2)
 *   bp_cache_apply        trainer-side cache maintenance: write back evicted rows, load prefetched rows
 *                         (Section 3.4 "Trainer"; the backing table stands in for the embedding servers)
 *   bp_embbag_fwd         EmbeddingBag-sum forward over cache slots (Section 2.1, embedding lookup)
 *   bp_embbag_bwd_update  deterministic backward + fused sparse optimizer step on cached rows
 *
 * Conventions
 *   - Every function returns BP_OK (0) or a negative bp_status.  bp_last_error_message() gives detail
 *     for the calling thread's last failure.
 *   - The library never allocates or frees device or pinned memory: inputs, outputs and workspaces are
 *     caller-owned and passed as raw pointers.  "device" below means a pointer the GPU can dereference
 *     (HBM, or pinned host memory from hipHostMalloc, which is device-visible at the same address);
 *     "host" means ordinary host memory read or written by the CPU inside the call.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null stream) of the
 *     current HIP device.  Only bp_oracle_plan synchronises the stream (it returns counts to the host).
 *   - Rows are `dim` elements of weight_dtype (fp32, or bf16 with fp32 arithmetic and
 *     round-to-nearest-even stores).  Row pointers must be 16-byte aligned and dim*sizeof(element)
 *     must be a multiple of 16 bytes for fp32 (dim % 4 == 0) and bf16 (dim % 8 == 0).
 *   - Optimizer state: BP_SGD none (pass NULL); BP_ADAGRAD fp32 [rows][dim]; BP_ADAGRAD_ROWWISE
 *     fp32 [rows].  The state of a cached row travels with the row.
 */
#ifndef BAGPIPE_H_
#define BAGPIPE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum bp_status {
    BP_OK = 0,
    BP_ERR_INVALID_ARG = -1,         /* NULL pointer, negative size, unsupported dim/dtype/optimizer */
    BP_ERR_CAPACITY = -2,            /* one batch's unique rows exceed the cache capacity */
    BP_ERR_WORKSPACE_TOO_SMALL = -3, /* workspace or list capacity below what the query function reports */
    BP_ERR_ID_OUT_OF_RANGE = -4,     /* an id outside [0, total_rows) */
    BP_ERR_HIP = -5,                 /* a HIP runtime call failed */
    BP_ERR_UNSUPPORTED = -6          /* size beyond a documented limit */
} bp_status;

/* How the planner's optional grouping cuts a batch's work for the backward pass (shared by the planner and the
 * backward kernels): a row looked up more than BP_BWD_ROW_MAX times in a batch is a "long row" and is handed out in
 * pieces of BP_BWD_PIECE lookups at most. */
#define BP_BWD_ROW_MAX 16
#define BP_BWD_PIECE 256

/* One distinct row of a batch, in the batch's grouped order (see bp_plan.grouped_lookups). */
typedef struct bp_row_rec {
    uint32_t start;   /* grouped position of the row's first lookup, counted from the batch's first grouped lookup;
                         bit 31 is set for a long row (more than BP_BWD_ROW_MAX lookups) */
    uint32_t count;   /* lookups of the row in this batch, >= 1 */
    int32_t slot;     /* the row's cache slot */
    uint32_t first;   /* lookup position (in the batch) of its first lookup == grouped_lookups[start] */
} bp_row_rec;

/* One piece of a long row: lookups [start, start + count) of the batch's grouped order. */
typedef struct bp_piece_rec {
    uint32_t start;    /* grouped position of the piece's first lookup (relative to the batch) */
    uint32_t count;    /* 1 .. BP_BWD_PIECE */
    int32_t slot;      /* the row's cache slot */
    uint32_t index;    /* which piece of its row, 0 .. pieces - 1 */
    uint32_t pieces;   /* pieces of the row: ceil(lookups of the row / BP_BWD_PIECE) */
    uint32_t partial;  /* rows of two or more pieces: the pieces of such rows are numbered through the batch in
                          grouped order from 0; this is the number of the row's piece 0 (undefined for one piece) */
    uint32_t reserved0, reserved1;
} bp_piece_rec;

enum { BP_F32 = 0, BP_BF16 = 1 };
enum { BP_SGD = 0, BP_ADAGRAD = 1, BP_ADAGRAD_ROWWISE = 2 };

/* Problem description, passed by pointer to every call (host memory, read during the call only). */
typedef struct bp_config {
    int64_t total_rows;   /* R: rows of the backing table; ids are global row numbers in [0, R) */
    int64_t capacity;     /* C: cache slots, 1 <= C < 2^31 (the paper's mandatory "max cache size", Section 4) */
    int32_t dim;          /* D */
    int32_t weight_dtype; /* BP_F32 | BP_BF16 */
    int32_t optimizer;    /* BP_SGD | BP_ADAGRAD | BP_ADAGRAD_ROWWISE */
    int32_t lookahead;    /* requested lookahead value: window of this many batches including the current
                             one (Algorithm 1's LookAheadValue), >= 1.  0 = not configured: the planner takes the
                             number of leading batches whose distinct rows together fit capacity - reserve slots
                             (the start-up rule of Section 4, "Automatically Calculating Lookahead": batches are
                             fetched ahead until no slot is left) and applies the capacity policy to it */
    float lr;             /* learning rate */
    float eps;            /* Adagrad epsilon */
    int64_t reserve;      /* slots the planner's capacity policy leaves free, 0 <= reserve < capacity: L_eff is the
                             largest lookahead whose peak occupancy is <= capacity - reserve, while slots still come
                             from all `capacity` slots.  With reserve >= the misses of any one batch, every slot a
                             batch's prefetches land in was already free before the previous batch trained, so they
                             can be fetched while that batch trains (Section 3.2: prefetching overlaps training). */
    int64_t cache_w_stride;     /* bytes from one row of cache_w to the next; 0 = dim * sizeof(element) (rows back to
                                   back); else a multiple of 16 that is at least that */
    int64_t cache_state_stride; /* the same for cache_state; 0 = the state's own size (dim * 4 bytes, or 4 for the
                                   row-wise rule); else a multiple of 16 (of 4 for the row-wise rule) that is at least
                                   that.  A caller that keeps a row's state right behind its weights allocates one
                                   array of capacity records of row + state bytes, passes cache_state = cache_w + row
                                   bytes and the record size as both strides: a 192-byte row and its 192-byte state
                                   then fill three whole 128-byte lines instead of touching four.  The backing table
                                   is always dense. */
} bp_config;

/* ------------------------------------------------------------------------------------------------
 * (1) Planner.  Algorithm 1 over a whole trace of T batches, plus the two choices the paper leaves
 * open: the effective lookahead L_eff is the largest L' <= lookahead whose peak cache occupancy is
 * <= capacity - reserve (Section 4, "Automatically Calculating Lookahead"), and cache slots come from a FIFO
 * ring of free slots (initially 0..C-1; misses of a batch pop in ascending id order, evictions push
 * in ascending id order after all pops of that batch).
 *
 * For batch i (0-based) with sorted distinct ids U_i the plan holds
 *   keep list      (id, ttl) for every id of U_i; ttl = last batch in [i, i+L_eff-1] that uses the id
 *   prefetch list  (id, slot) for the ids of U_i not resident before batch i
 *   evict list     (id, slot) for the ids of U_i with ttl == i, to be written back after batch i
 *   lookup_slots   cache slot of every lookup of the trace, in lookup order
 * all lists ascending in id inside a batch, concatenated over batches (CSR offsets on the host).
 * ------------------------------------------------------------------------------------------------ */
typedef struct bp_plan {
    /* device outputs, caller-allocated */
    int32_t* lookup_slots;    /* [n_lookups]; may be NULL when the grouping outputs below are asked for: a caller that
                                 walks the row records (bp_embbag_fwd_grouped, bp_embbag_bwd_update_grouped) needs no
                                 slot per lookup, and the planner then saves the pass that scatters them */
    int64_t* prefetch_ids;    /* [list_capacity] */
    int32_t* prefetch_slots;  /* [list_capacity] */
    int64_t* evict_ids;       /* [list_capacity] */
    int32_t* evict_slots;     /* [list_capacity] */
    int64_t* keep_ids;        /* [list_capacity] */
    int32_t* keep_ttl;        /* [list_capacity] */
    int64_t list_capacity;    /* entries each list can hold; n_lookups is always enough, sum_i |U_i| is needed */
    /* host outputs, caller-allocated */
    int64_t* prefetch_offsets; /* [T+1] */
    int64_t* evict_offsets;    /* [T+1] */
    int64_t* keep_offsets;     /* [T+1] */
    int64_t* occupancy;        /* [T] rows resident while batch i trains */
    /* optional (all four NULL, or all four set): every batch's lookups grouped by row, which is a by-product of the
     * planner's sort and lets bp_embbag_bwd_update_grouped skip its own sort.  Inside a batch the lookups are
     * ordered by id ascending and, for one id, by lookup position ascending; the batch's distinct rows, in that
     * order, are its keep-list entries, and row_recs is parallel to the keep list. */
    int32_t* grouped_lookups;  /* device [n_lookups] position of each grouped lookup, relative to the batch's first lookup */
    bp_row_rec* row_recs;      /* device [list_capacity], entry k describes the row of keep-list entry k
                                  (keep_offsets are its CSR offsets too) */
    bp_piece_rec* piece_recs;  /* device [n_lookups / (BP_BWD_ROW_MAX + 1) + n_lookups / BP_BWD_PIECE + 2]: the pieces of
                                  every long row, rows in grouped order, pieces of a row in order */
    int64_t* piece_offsets;    /* host [T+1] CSR offsets of the batches into piece_recs */
    /* optional: which logical trainer uses a row (Section 3.3: rows used by a single trainer need no synchronisation;
     * of the shared rows only those the next batch needs are synchronised on the critical path).  All three set or
     * none.  The lookups of batch i are dealt to n_trainers trainers by position: trainer t owns the positions
     * [trainer_cuts[i*(n_trainers+1) + t], trainer_cuts[i*(n_trainers+1) + t + 1]) counted from the batch's first
     * lookup (non-decreasing, from 0 to the batch's size). */
    const int64_t* trainer_cuts;   /* input, host [T][n_trainers + 1] */
    int32_t n_trainers;            /* input, 1 .. 64 */
    int32_t* keep_owner;           /* output, device [list_capacity], parallel to keep_ids: t when only trainer t looks
                                      the id up in that batch; -1 several trainers and the next batch does not use
                                      it; -2 several trainers and the next batch uses it too */
    /* scalar results */
    int32_t L_eff;
    int32_t L_requested;       /* the lookahead the capacity policy started from: cfg->lookahead, or, when that is 0,
                                  the start-up rule's value (see bp_config.lookahead) */
    int64_t peak_occupancy;
    int64_t min_capacity;      /* max_i |U_i|: the smallest capacity - reserve for which a plan exists */
    int64_t n_unique_pairs;    /* sum_i |U_i| */
} bp_plan;

/* Bytes of device workspace bp_oracle_plan needs for a trace of n_lookups lookups in n_iters batches;
 * with_grouping != 0 when the plan's optional grouping outputs are requested. */
int bp_oracle_plan_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int32_t n_iters, int32_t with_grouping,
                                   size_t* bytes);

/*
 * ids          device, [n_lookups] global row ids in lookup order, batches concatenated
 * iter_offsets host, [n_iters+1], non-decreasing, iter_offsets[0] == 0, last == n_lookups
 * plan         host struct; its pointers as documented above; scalars are written on return
 * workspace    device, at least bp_oracle_plan_workspace_bytes() bytes, 256-byte aligned
 * Limits: n_lookups < 2^31, 1 <= n_iters <= 8192, bits(total_rows) + 2 * bits(n_iters) + 2 <= 64 and
 * max(bits(total_rows), 32) + bits(n_iters) + bits(lookups of the largest batch) <= 64 (bits(x) = bits needed for
 * values below x; a lookup travels as one 64-bit word of id or slot, batch and place in the batch), else
 * BP_ERR_UNSUPPORTED.
 * Errors: BP_ERR_ID_OUT_OF_RANGE; BP_ERR_CAPACITY (plan->min_capacity is set); BP_ERR_WORKSPACE_TOO_SMALL
 * (also when list_capacity < n_unique_pairs; plan->n_unique_pairs is set).  On error the device outputs
 * are unspecified.  Synchronises `stream`.
 */
int bp_oracle_plan(const bp_config* cfg, const int64_t* ids, const int64_t* iter_offsets, int32_t n_iters,
                   bp_plan* plan, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Chunked planning for a stream of batches (the paper's Oracle Cacher sees the batches as they arrive, a lookahead
 * ahead of the trainers, Sections 3.1 and 3.3): bp_oracle_plan_chunk plans the first n_emit of the n_iters batches
 * it is given and carries the state of the cache to the next call.  The batches after the n_emit-th are the window
 * the decisions look into: pass min(lookahead - 1, what the stream still holds) of them.  With the same effective
 * lookahead in every chunk the concatenated plans equal bp_oracle_plan's over the whole stream, slot for slot.
 * The capacity policy is applied per chunk, so the effective lookahead may change from chunk to chunk; a row kept
 * under an earlier, larger lookahead stays until its next use.  The policy looks at every batch the chunk's
 * decisions reach, not only at the emitted ones: the batches of the window count too (each held to
 * capacity - reserve rows with the chunk's lookahead behind it and a lookahead of one from there on), so that a chunk
 * never leaves its successor a cache it cannot plan.  Consequently BP_ERR_CAPACITY, or a lowered L_eff, may be due
 * to a batch of the window.
 *
 * bp_plan_state   n_resident rows are in the cache at the boundary: resident_ids (device [capacity], ascending)
 *                 and ring (device [capacity]): the residents' slots in the same order, then the free slots in
 *                 the order they will be handed out.  state_in == NULL: empty cache, slots 0..capacity-1 in order.
 *                 state_in and state_out must be different buffers; the caller owns both.
 * plan            as for bp_oracle_plan, with these differences: host arrays have n_emit + 1 (offsets) or n_emit
 *                 (occupancy) entries; offsets are positions in the device lists and need not start at 0 (the carried
 *                 rows' own entries come first); keep_ttl counts batches from the chunk's first batch; lookup_slots
 *                 and the grouping cover all n_iters batches given, but past the n_emit-th batch their contents are
 *                 unspecified (slots may be -1 there: the window is planned without a bound on its occupancy);
 *                 list_capacity >= n_unique_pairs, which counts the carried rows too; peak_occupancy and
 *                 min_capacity are taken over all n_iters batches given, window included: peak_occupancy counts, in
 *                 a batch of the window, its own rows and what this chunk's decisions and the carried rows leave
 *                 there; min_capacity is the smallest capacity - reserve that admits a lookahead of one (a batch's
 *                 distinct rows plus the carried rows still held over it).
 * workspace       bp_oracle_plan_chunk_workspace_bytes(cfg, n_lookups, n_iters, with_grouping) bytes.
 * Errors as for bp_oracle_plan.  Synchronises `stream`.
 */
typedef struct bp_plan_state {
    int64_t n_resident;
    int64_t* resident_ids;
    int32_t* ring;
} bp_plan_state;
int bp_oracle_plan_chunk_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int32_t n_iters, int32_t with_grouping,
                                         size_t* bytes);
int bp_oracle_plan_chunk(const bp_config* cfg, const int64_t* ids, const int64_t* iter_offsets, int32_t n_iters,
                         int32_t n_emit, const bp_plan_state* state_in, bp_plan_state* state_out, bp_plan* plan,
                         void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * (2) Cache maintenance between two batches: first every evicted row (weights and optimizer state) is
 * copied from its cache slot back to the backing table, then every prefetched row is copied from the
 * backing table into its slot — in that order, so a slot freed by an eviction may be refilled in the
 * same call, and a row is only fetched after its last update was written back (Section 3.2,
 * "Consistency with the Lookahead algorithm").
 *
 * cache_w / cache_state     device (HBM), [capacity] rows (strides: bp_config.cache_w_stride / cache_state_stride)
 * backing_w / backing_state device-visible backing table [total_rows] rows (pinned host memory, or HBM)
 * evict_* / prefetch_*      device, list slices of one batch from bp_plan; n_* may be 0 (pointers then unused)
 * Entries with id or slot out of range are skipped.  Asynchronous on `stream`.
 * ------------------------------------------------------------------------------------------------ */
int bp_cache_apply(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                   const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict,
                   const int64_t* prefetch_ids, const int32_t* prefetch_slots, int64_t n_prefetch, void* stream);

/*
 * The same maintenance with both directions of the host link busy at once.  Evicted rows are first copied to a
 * staging area in HBM (which frees their slots), then ONE launch writes the staged rows to the backing table while
 * it reads the prefetched rows from it.  Precondition: no id is in both lists — true for every plan with
 * L_eff >= 2 (a row evicted after batch i-1 is not used by batch i); with L_eff == 1 use bp_cache_apply.
 * The result is then identical to bp_cache_apply.
 *
 * workspace  device (HBM), bp_cache_apply_duplex_workspace_bytes(cfg, n_evict) bytes, 256-byte aligned; unused when
 *            n_evict == 0
 * Other arguments and error behaviour as for bp_cache_apply.  Asynchronous on `stream`.
 */
int bp_cache_apply_duplex_workspace_bytes(const bp_config* cfg, int64_t n_evict, size_t* bytes);
int bp_cache_apply_duplex(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                          const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict,
                          const int64_t* prefetch_ids, const int32_t* prefetch_slots, int64_t n_prefetch,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two halves of bp_cache_apply_duplex as calls of their own, for a schedule that overlaps cache maintenance with
 * training (Section 3.2 and 3.4: prefetches and write-backs run beside the trainer, touching slots the running batch
 * does not use):
 *   bp_cache_stage         copies the evicted rows (weights, state) from their slots to the staging area, entry e to
 *                          staging row e; afterwards the slots may be refilled.
 *   bp_cache_apply_staged  ONE launch writes the staged rows to the backing table (entry e to row evict_ids[e]) and
 *                          copies the prefetched rows from the backing table into their slots.  Precondition: no id
 *                          is in both lists.  Either list may be empty.
 * Both calls of a pair take the same evict list and n_evict (the staging layout depends on n_evict) and the same
 * staging area: device (HBM), bp_cache_apply_duplex_workspace_bytes(cfg, n_evict) bytes, 256-byte aligned, unused
 * when n_evict == 0.  Entries with id or slot out of range are skipped by both.  Asynchronous on `stream`.
 */
int bp_cache_stage(const bp_config* cfg, const void* cache_w, const void* cache_state, const int32_t* evict_slots,
                   int64_t n_evict, void* staging, size_t staging_bytes, void* stream);
int bp_cache_apply_staged(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                          const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict, const void* staging,
                          size_t staging_bytes, const int64_t* prefetch_ids, const int32_t* prefetch_slots,
                          int64_t n_prefetch, void* stream);

/*
 * The same maintenance in ONE launch and without a staging area, for lists that come from the planner's FIFO ring:
 * there the prefetches of a batch that land in slots freed by the previous batch's evictions are the last
 * n_prefetch - n_early entries of the prefetch list and take those slots in the evictions' own order (prefetch entry
 * n_early + k gets the slot of evict entry k), so one lane group moves the evicted row out of a slot and the fetched
 * row into it, one after the other.  n_early = the leading prefetch entries whose slots were free before: for batch
 * i of a whole-trace plan, clamp(capacity + evict_offsets[i-1] - prefetch_offsets[i], 0, misses of i) (the evictions
 * are those of batch i-1; evict_offsets[i-1] counts the evictions of the batches before it).
 * Preconditions: no id in both lists (L_eff >= 2), and the pairing above.  A pair whose slots differ is left alone
 * (its slot keeps the evicted row, which is still written back) and *mismatch_flag (device, may be NULL; the caller
 * clears it) is set to 1: a set flag means the cache is not what the plan says.
 * Other arguments and error behaviour as for bp_cache_apply.  Asynchronous on `stream`.
 */
int bp_cache_apply_handoff(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                           const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict,
                           const int64_t* prefetch_ids, const int32_t* prefetch_slots, int64_t n_prefetch,
                           int64_t n_early, uint32_t* mismatch_flag, void* stream);

/* ------------------------------------------------------------------------------------------------
 * (2b) Cache maintenance overlapped with training (Section 3.2: the lookahead lets rows be fetched before the
 * batch that needs them; Section 3.4: the trainer's cache is maintained beside the training step, on slots the
 * running batch does not touch).  A bp_pipeline owns a maintenance stream and enqueues, for a plan of T batches,
 *     after batch i:  A_i  stage the rows evicted after batch i; fetch the late prefetches of batch i+1
 *                     B_i  write the staged rows back; fetch the early prefetches of batch i+2
 * where the EARLY prefetches of batch j are the leading entries of its prefetch list whose slot was already free
 * before batch j-1 (their count follows from the FIFO ring: capacity + evictions of batches <= j-2 - misses of
 * batches < j, clamped to [0, misses of j]; zero when L_eff < 2 and for batch 0).  B_i runs while batch i+1
 * trains.  The result (cache, backing table) is the one of the synchronous order of (2).
 *
 * Use:  create; begin(compute_stream); for every batch i in order: acquire(i, cs), the caller's forward and
 * backward/update of batch i on cs, release(i, cs); end(cs); destroy.
 *   create   copies the host offsets; the device lists (slices of a bp_plan), the cache, the backing table and the
 *            staging area (device, bp_cache_apply_duplex_workspace_bytes(cfg, largest evict list) bytes, 256-byte
 *            aligned) must stay valid until destroy.  Creates one stream (default priority) and five events.
 *   begin    orders the maintenance stream behind everything enqueued on compute_stream so far, then enqueues the
 *            fetches for batch 0 and the early ones for batch 1.
 *   acquire  makes compute_stream wait until batch i's rows are in the cache.
 *   release  makes the maintenance stream wait for what compute_stream has enqueued so far (batch i's update),
 *            then enqueues A_i and B_i.
 *   end      makes compute_stream wait for all maintenance work (the last write-backs).
 *   destroy  waits for the maintenance stream and frees the object; NULL is allowed.
 * All calls are host-side and asynchronous except destroy.  One pipeline serves one pass over its plan; begin may
 * be called again after end.  bp_pipeline_early_counts is the host-only computation of the early counts
 * (early[n_iters], no GPU call); bp_pipeline_early reads one of them back.
 * ------------------------------------------------------------------------------------------------ */
typedef struct bp_pipeline bp_pipeline;
int bp_pipeline_early_counts(const int64_t* prefetch_offsets, const int64_t* evict_offsets, int32_t n_iters,
                             int64_t capacity, int32_t L_eff, int64_t* early);
int bp_pipeline_create(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                       const int64_t* prefetch_ids, const int32_t* prefetch_slots, const int64_t* prefetch_offsets,
                       const int64_t* evict_ids, const int32_t* evict_slots, const int64_t* evict_offsets,
                       int32_t n_iters, int32_t L_eff, void* staging, size_t staging_bytes, bp_pipeline** out);
int bp_pipeline_destroy(bp_pipeline* p);
int bp_pipeline_early(const bp_pipeline* p, int32_t batch, int64_t* early);
int bp_pipeline_begin(bp_pipeline* p, void* compute_stream);
int bp_pipeline_acquire(bp_pipeline* p, int32_t batch, void* compute_stream);
int bp_pipeline_release(bp_pipeline* p, int32_t batch, void* compute_stream);
int bp_pipeline_end(bp_pipeline* p, void* compute_stream);

/* ------------------------------------------------------------------------------------------------
 * (3) Forward: out[b, :] = sum over lookups k in [bag_offsets[b], bag_offsets[b+1]) of cache_w[slot[k], :],
 * accumulated in fp32 in lookup order; an empty bag gives a zero row.
 *
 * lookup_slots device, [n_lookups] slots of this batch's lookups (a slice of bp_plan.lookup_slots)
 * bag_offsets  device, [bags+1] int64 starting at 0 and ending at n_lookups; NULL means one lookup per bag
 *              (n_lookups == bags)
 * out          device, fp32 [bags][dim]
 * Slots outside [0, capacity) contribute nothing.  Asynchronous on `stream`.
 * ------------------------------------------------------------------------------------------------ */
int bp_embbag_fwd(const bp_config* cfg, const void* cache_w, const int32_t* lookup_slots,
                  const int64_t* bag_offsets, int64_t n_lookups, int64_t bags, float* out, void* stream);

/*
 * The forward pass of a batch with ONE lookup per bag, walked by the plan's grouping instead of a slot per lookup:
 * every row record's row is fetched once and written to out[b, :] for every bag b among the row's grouped lookups
 * (one lane group per row of up to BP_BWD_ROW_MAX lookups, one workgroup per piece of a longer row).  With a
 * grouping that holds its contract every bag is named once and `out` equals bp_embbag_fwd's bit for bit; a bag that
 * no record names keeps whatever `out` held.
 *
 * grouped_lookups      device, the batch's slice [iter_offsets[i], iter_offsets[i+1]) of the plan array ([bags])
 * row_recs, n_rows     device, the batch's slice [keep_offsets[i], keep_offsets[i+1]) and its length
 * piece_recs, n_pieces device, the batch's slice [piece_offsets[i], piece_offsets[i+1]) and its length (may be 0)
 * Records that point outside the batch, bags outside [0, bags) and slots outside [0, capacity) write nothing.
 * Limits and error behaviour as for bp_embbag_fwd.  Asynchronous on `stream`.
 */
int bp_embbag_fwd_grouped(const bp_config* cfg, const void* cache_w, const int32_t* grouped_lookups,
                          const bp_row_rec* row_recs, int64_t n_rows, const bp_piece_rec* piece_recs, int64_t n_pieces,
                          int64_t bags, float* out, void* stream);

/* ------------------------------------------------------------------------------------------------
 * (4) Backward + update, deterministic (bit-identical from run to run): lookups are grouped by slot with
 * a stable radix sort, the same row and piece records as the planner's grouping are built on the device,
 * G[slot, :] = sum of grad_out[bag(k), :] over the slot's lookups is formed in a
 * fixed order with fp64 accumulators and rounded once to fp32, and each distinct slot is updated once,
 * in place, in fp32 arithmetic (one rounding per operation, no fused multiply-add):
 *   BP_SGD              w -= lr * G
 *   BP_ADAGRAD          s += G*G;              w -= lr * G / (sqrt(s) + eps)
 *   BP_ADAGRAD_ROWWISE  s_row += mean_d G_d^2; w -= lr * G / (sqrt(s_row) + eps)
 * (gradients of duplicate lookups are added before squaring; any optimizer of this form works because
 * gradients, not embeddings, are combined — Section 6.)
 *
 * grad_out   device, fp32 [bags][dim]
 * workspace  device, at least bp_embbag_bwd_update_workspace_bytes() bytes, 256-byte aligned
 * tickets    device, at least bp_embbag_bwd_ticket_bytes(n_lookups) bytes of counters (uint32), ALL ZERO when the call
 *            starts its work on `stream`.  The call leaves them all zero again when that work has finished, so one
 *            buffer sized for the largest batch, zeroed once when it is allocated, serves every later call on the
 *            same stream (calls that overlap in time need buffers of their own).  They count, for a row whose
 *            lookups are spread over several workgroups, how many of those have stored their sum.
 * Limits: n_lookups < 2^31, bags < 2^31.  Slots outside [0, capacity) are ignored.  Asynchronous.
 * ------------------------------------------------------------------------------------------------ */
int bp_embbag_bwd_update_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int64_t bags, size_t* bytes);
size_t bp_embbag_bwd_ticket_bytes(int64_t n_lookups);
int bp_embbag_bwd_update(const bp_config* cfg, void* cache_w, void* cache_state, const int32_t* lookup_slots,
                         const int64_t* bag_offsets, int64_t n_lookups, int64_t bags, const float* grad_out,
                         void* workspace, size_t workspace_bytes, uint32_t* tickets, void* stream);

/*
 * The same backward + update for a batch whose lookups the plan has already grouped by row (bp_plan's
 * optional outputs): no sort and no scan at run time, ONE kernel launch (three when bag_offsets is given).  A row of
 * up to BP_BWD_ROW_MAX lookups is summed and updated by one lane group; every piece of a long row by one workgroup,
 * and a row of several pieces is finished by whichever of its workgroups ends last, which adds the pieces' sums in
 * piece order.  Results are those of bp_embbag_bwd_update up to the order in which a row's gradients enter the
 * fp64 sum; that order is fixed by the records, never by timing.
 *
 * grouped_lookups     device, the batch's slice [iter_offsets[i], iter_offsets[i+1]) of the plan array
 * row_recs, n_rows    device, the batch's slice [keep_offsets[i], keep_offsets[i+1]) and its length
 * piece_recs, n_pieces device, the batch's slice [piece_offsets[i], piece_offsets[i+1]) and its length (may be 0)
 * workspace           device, bp_embbag_bwd_update_grouped_workspace_bytes() bytes (multi_hot != 0 when bag_offsets is
 *                     not NULL), 256-byte aligned
 * tickets             as for bp_embbag_bwd_update: zeroed counters, left zero
 * Records that point outside the batch or the workspace are skipped.  Other arguments, limits and error behaviour
 * as for bp_embbag_bwd_update.  Asynchronous.
 */
int bp_embbag_bwd_update_grouped_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int64_t bags,
                                                 int32_t multi_hot, size_t* bytes);
int bp_embbag_bwd_update_grouped(const bp_config* cfg, void* cache_w, void* cache_state, const int32_t* grouped_lookups,
                                 const bp_row_rec* row_recs, int64_t n_rows, const bp_piece_rec* piece_recs,
                                 int64_t n_pieces, const int64_t* bag_offsets, int64_t n_lookups, int64_t bags,
                                 const float* grad_out, void* workspace, size_t workspace_bytes, uint32_t* tickets,
                                 void* stream);

/*
 * bp_embbag_bwd_update_grouped for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments without workspace and tickets: both live in a
 * fixed array of bp_embbag_bwd_update_grouped_static_max_bytes() bytes (16 MiB) in device memory that belongs to the
 * library (every GPU the library has run this call on holds its own copy until the process ends).  The call
 * allocates and frees nothing; the first call on a device looks the array's address up and clears it with one small
 * kernel on `stream`.  A batch whose scratch (bp_embbag_bwd_update_grouped_static_bytes) does not fit is refused with
 * BP_ERR_UNSUPPORTED.  All calls on one GPU share the array: calls that overlap in time on one GPU race; calls on
 * one stream, or ordered by events, do not.  Results are those of bp_embbag_bwd_update_grouped, bit for bit.
 */
size_t bp_embbag_bwd_update_grouped_static_max_bytes(void);
int bp_embbag_bwd_update_grouped_static_bytes(const bp_config* cfg, int64_t n_lookups, int64_t bags, int32_t multi_hot,
                                              size_t* bytes);
int bp_embbag_bwd_update_grouped_static(const bp_config* cfg, void* cache_w, void* cache_state,
                                        const int32_t* grouped_lookups, const bp_row_rec* row_recs, int64_t n_rows,
                                        const bp_piece_rec* piece_recs, int64_t n_pieces, const int64_t* bag_offsets,
                                        int64_t n_lookups, int64_t bags, const float* grad_out, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Diagnostics.
 * ------------------------------------------------------------------------------------------------ */
/* Plain device-to-device copy of `bytes` bytes (multiple of 16, 16-byte aligned pointers) by a streaming kernel:
 * a yardstick of known size for hardware byte counters and for achievable copy bandwidth.  Asynchronous. */
int bp_copy_calibration(void* dst, const void* src, size_t bytes, void* stream);
/* Reads the n rows `rows[k]` (device uint32; a number >= table_rows reads the last row) of a device table of
 * table_rows rows of row_bytes bytes each (multiple of 16, at most 1024; 16-byte aligned) and folds them into
 * `sink` (device, 16 bytes per lane group: 16 * (ceil(n / rows_in_flight) + 256) bytes): lane groups take
 * rows_in_flight (1, 2, 4 or 8) consecutive entries of `rows` each, all their loads in flight together; four is how
 * the backward pass reads gradient rows.  A yardstick for the rate at which randomly placed rows can be fetched with
 * nothing else going on.  Asynchronous. */
int bp_gather_calibration(void* sink, const void* table, int64_t table_rows, int32_t row_bytes, const uint32_t* rows,
                          int64_t n, int32_t rows_in_flight, void* stream);

/* Writes the n rows `rows[k]` (device uint32; a number >= table_rows is skipped; a row listed twice keeps either
 * writer's pieces) of a device table of table_rows rows of row_bytes bytes each (multiple of 16, at most 1024; 16-byte
 * aligned), rows_in_flight (1, 2 or 4) list entries per lane group, reading nothing but the list: the 16-byte piece
 * c of row r written for list entry k holds the uint32 words {r, c, k, 0x5ca77e25}.  A yardstick for the rate at
 * which randomly placed rows can be written with nothing else going on, which bounds the forward pass over one-lookup
 * bags (one output row per lookup).  Asynchronous. */
int bp_scatter_calibration(void* table, int64_t table_rows, int32_t row_bytes, const uint32_t* rows, int64_t n,
                           int32_t rows_in_flight, void* stream);

const char* bp_error_string(int status);
const char* bp_last_error_message(void);   /* thread-local, valid until the thread's next failing call */
int bp_version(void);

/*
 * Per-kernel timing with HIP events: every profiled launch carries a start and a stop event of its own, stamped by
 * the runtime with the kernel's begin and end on the launch stream.
 * bp_profile_enable(1) starts recording (and clears old records); bp_profile_enable(0) stops.
 * bp_profile_collect() synchronises the recorded events and adds their durations to per-kernel totals;
 * bp_profile_get() reads the totals of kernel `id` in [0, bp_profile_num_kernels()).
 * bp_profile_select(mask) restricts recording to the kernels whose id bit is set (default: all), so that a
 * timed loop can bracket one kernel only and pay two event records per launch of that kernel.
 * Recording creates HIP events (no device memory).  Not thread-safe.
 */
int bp_profile_enable(int on);
int bp_profile_select(uint64_t kernel_mask);
/* Median reading, in microseconds, of the same pair of events around a kernel that does nothing (`reps` launches on
 * `stream`, synchronises it): the share of every profiled duration that is the bracket, not the kernel. */
int bp_profile_bracket_overhead(void* stream, int32_t reps, double* median_us);
int bp_profile_collect(void);
/* Shortest, median and longest launch of kernel `id` among those collected since bp_profile_enable(1), in ms
 * (BP_ERR_INVALID_ARG when none was recorded). */
int bp_profile_spread(int id, double* min_ms, double* median_ms, double* max_ms);
int bp_profile_num_kernels(void);
const char* bp_profile_kernel_name(int id);
int bp_profile_get(int id, int64_t* launches, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* BAGPIPE_H_ */
