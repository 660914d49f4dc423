/*
 * CPU oracle for the embedding-access hot path of lookahead-cached recommendation-model training.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU library is checked
 * against.  It shares no code with the GPU library, and nothing in the product path may call it:
 * only tests, the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * Three parts:
 *   A. the lookahead planner (Algorithm 1 and Section 3.2 of the paper).  What it decides, in this
 *      file's own terms: batch i looks into the window of batches [i, i + L - 1]; an id of batch i is
 *      kept until its last use inside that window (its TTL) and written back after the batch whose
 *      number equals that TTL; an id that is not resident when its batch comes up is fetched.  The
 *      per-id bookkeeping is two arrays indexed by id (last batch of the window that uses the id;
 *      resident or not / slot).  Two things the paper leaves open are fixed here:
 *        - capacity policy (Section 4, "Automatically Calculating Lookahead": the lookahead is reduced
 *          when the cache would overflow): the effective lookahead is the largest L' <= L whose peak
 *          occupancy fits in the cache;
 *        - slot assignment (Section 4, "Overlapping cache management with training" only says that
 *          trainer and maintenance touch disjoint indices): a FIFO ring of free slots.
 *   B. uncached synchronous training on the full table: EmbeddingBag sum forward, gradient coalescing,
 *      SGD / Adagrad update (the paper's statement that training matches synchronous baselines,
 *      Section 5, paragraph "Metrics", and Section 5.1 "Convergence Comparison", makes this the definition of the right answer).
 *   C. the same arithmetic routed through the plan and a cache array with write-backs.
 *
 * Floating point: rows are stored in their storage type (fp32, or bf16 with round-to-nearest-even).
 * Every sum is carried out in fp64.  With fp32 storage the update is carried out in fp64 too and rounded
 * once on store; with bf16 storage the stored value is a quantised code and the update is carried out in
 * fp32, the arithmetic type fixed for that workload (see update_row_bf16).
 * Parity pins: tests/test_oracle_*.py (paper's worked example, brute force from the plain
 * definitions, invariants, torch CPU library routines).  Row-wise Adagrad is pinned, for fp32 and for
 * bf16 rows, by hand-computed one-row values, by its equality with element-wise Adagrad at D = 1,
 * against torch's Adagrad on gradients that are constant along a row, and against the same rule written
 * with torch tensor operations on gradients that vary along a row (several rows, several steps).
 * Further parts, each with its own pins: the lookahead when none is configured (orc_auto_lookahead),
 * a lookahead that changes from batch to batch (orc_plan_stream), the trainers that use a row
 * (orc_keep_owners), and a multi-threaded leg of the training iteration (orc_train_iter_mt: same
 * arithmetic in the same order per bag and per row, pinned bit for bit against the serial routine).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_CAPACITY (-2)
#define ORC_ERR_ID_RANGE (-3)
#define ORC_ERR_NOMEM (-4)
#define ORC_ERR_INTERNAL (-5)

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_SGD = 0, ORC_ADAGRAD = 1, ORC_ADAGRAD_ROWWISE = 2 };

/* ------------------------------------------------------------------ helpers */
static int cmp_i64(const void *a, const void *b) {
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

/*
 * The distinct ids of every batch (what Algorithm 1 iterates over), sorted.
 * uniq must hold N entries; uniq_off[T+1] receives the CSR offsets.  Returns total count or <0.
 */
int64_t orc_unique_per_iter(const int64_t *ids, const int64_t *iter_off, int64_t T, int64_t total_rows,
                            int64_t *uniq, int64_t *uniq_off) {
    int64_t w = 0;
    uniq_off[0] = 0;
    for (int64_t i = 0; i < T; ++i) {
        int64_t a = iter_off[i], b = iter_off[i + 1], s = w;
        for (int64_t k = a; k < b; ++k) {
            if (ids[k] < 0 || ids[k] >= total_rows) return ORC_ERR_ID_RANGE;
            uniq[w++] = ids[k];
        }
        qsort(uniq + s, (size_t)(w - s), sizeof(int64_t), cmp_i64);
        int64_t o = s;
        for (int64_t k = s; k < w; ++k)
            if (k == s || uniq[k] != uniq[k - 1]) uniq[o++] = uniq[k];
        w = o;
        uniq_off[i + 1] = w;
    }
    return w;
}

/* ------------------------------------------------------------------ part A: planner */

/*
 * Residency under Algorithm 1 with lookahead value Lp and no capacity limit.
 * occ[i] = number of embeddings in the cache while batch i trains (after its prefetches, before its
 * evictions).  Returns the peak, or <0 on error.
 *
 * The window always holds consecutive batches, so it is kept as the index range [i, pushed).
 * latest[id] = last batch of the window seen so far that uses the id; in_cache[id] = resident or not.
 */
int64_t orc_peak_occupancy(const int64_t *uniq, const int64_t *uniq_off, int64_t T, int64_t total_rows,
                           int64_t Lp, int64_t *occ) {
    if (Lp < 1 || T < 0) return ORC_ERR_ARG;
    int32_t *latest = (int32_t *)malloc((size_t)total_rows * sizeof(int32_t));
    uint8_t *in_cache = (uint8_t *)calloc((size_t)total_rows, 1);
    if (!latest || !in_cache) { free(latest); free(in_cache); return ORC_ERR_NOMEM; }
    int64_t pushed = 0, resident = 0, peak = 0;
    for (int64_t i = 0; i < T; ++i) {
        /* fill the queue up to Lp batches, recording the latest iteration each id occurs in */
        while (pushed < T && pushed - i < Lp) {
            for (int64_t k = uniq_off[pushed]; k < uniq_off[pushed + 1]; ++k) latest[uniq[k]] = (int32_t)pushed;
            ++pushed;
        }
        /* current batch = front of the queue: fetch what is not cached */
        for (int64_t k = uniq_off[i]; k < uniq_off[i + 1]; ++k) {
            int64_t g = uniq[k];
            if (!in_cache[g]) { in_cache[g] = 1; ++resident; }
        }
        if (occ) occ[i] = resident;
        if (resident > peak) peak = resident;
        /* after training: drop the ids whose TTL is the current batch */
        for (int64_t k = uniq_off[i]; k < uniq_off[i + 1]; ++k) {
            int64_t g = uniq[k];
            if (latest[g] == i) { in_cache[g] = 0; --resident; }
        }
    }
    free(latest); free(in_cache);
    return peak;
}

/*
 * Capacity policy: the largest L' in [1, L] with peak occupancy <= C.
 * exhaustive != 0: try L, L-1, ... one by one (the definition).
 * exhaustive == 0: bisection, valid because the set resident under L' is a subset of the set resident
 * under L'+1 at every iteration (an id stays iff its next use is fewer than L' batches ahead), so the
 * peak is non-decreasing in L'.  tests compare the two.
 * Returns L_eff, or ORC_ERR_CAPACITY when even L' = 1 does not fit (*min_capacity = max_i u_i then).
 */
int64_t orc_choose_lookahead(const int64_t *uniq, const int64_t *uniq_off, int64_t T, int64_t total_rows,
                             int64_t L, int64_t C, int exhaustive, int64_t *min_capacity) {
    if (L < 1 || C < 1) return ORC_ERR_ARG;
    int64_t p1 = orc_peak_occupancy(uniq, uniq_off, T, total_rows, 1, NULL);
    if (p1 < 0) return p1;
    if (min_capacity) *min_capacity = p1;
    if (p1 > C) return ORC_ERR_CAPACITY;
    int64_t Ltop = L < T ? L : (T > 0 ? T : 1);        /* windows of T or more batches are all the same */
    int64_t ptop = orc_peak_occupancy(uniq, uniq_off, T, total_rows, Ltop, NULL);
    if (ptop < 0) return ptop;
    if (ptop <= C) return L;
    if (exhaustive) {
        for (int64_t Lp = Ltop - 1; Lp >= 1; --Lp) {
            int64_t p = orc_peak_occupancy(uniq, uniq_off, T, total_rows, Lp, NULL);
            if (p < 0) return p;
            if (p <= C) return Lp;
        }
        return ORC_ERR_INTERNAL;
    }
    int64_t lo = 1, hi = Ltop;                         /* peak(lo) <= C < peak(hi) */
    while (hi - lo > 1) {
        int64_t mid = lo + (hi - lo) / 2;
        int64_t p = orc_peak_occupancy(uniq, uniq_off, T, total_rows, mid, NULL);
        if (p < 0) return p;
        if (p <= C) lo = mid; else hi = mid;
    }
    return lo;
}

/*
 * Lookahead when none is configured (Section 4, "Automatically Calculating Lookahead"): at start-up the batches are
 * prefetched one after the other until the cache is full; the number of batches prefetched by then is the lookahead.
 * Written out: the largest k such that the distinct ids of batches 0 .. k-1 together fit into C slots (k <= T).
 * Returns k (0 when even the first batch does not fit).
 */
int64_t orc_auto_lookahead(const int64_t *uniq, const int64_t *uniq_off, int64_t T, int64_t total_rows, int64_t C) {
    if (C < 1 || T < 0) return ORC_ERR_ARG;
    uint8_t *seen = (uint8_t *)calloc((size_t)(total_rows > 0 ? total_rows : 1), 1);
    if (!seen) return ORC_ERR_NOMEM;
    int64_t held = 0, k = 0;
    for (int64_t i = 0; i < T; ++i) {
        for (int64_t q = uniq_off[i]; q < uniq_off[i + 1]; ++q) {
            int64_t g = uniq[q];
            if (g < 0 || g >= total_rows) { free(seen); return ORC_ERR_ID_RANGE; }
            if (!seen[g]) { seen[g] = 1; ++held; }
        }
        if (held > C) break;
        k = i + 1;
    }
    free(seen);
    return k;
}

/*
 * The plan: Algorithm 1 with lookahead Leff, cache slots from a FIFO ring of C free slots.
 *
 * Per iteration i (two phases, so that a slot freed by one id of batch i is never handed to another
 * id of the same batch):
 *   phase 1, ids of the batch in ascending order: TTL = latest[id]; append (id, TTL) to the
 *            keep list; if the id is not cached, pop a slot from the ring head and append (id, slot)
 *            to the prefetch list;
 *   every lookup of the batch gets the slot of its id;
 *   phase 2, ids in ascending order: if TTL == i, append (id, slot) to the evict list, push the slot
 *            at the ring tail, erase the id.
 * Lists are CSR over iterations.  keep_* hold sum(u_i) entries; prefetch_* / evict_* hold at most that.
 * Returns number of prefetch entries (== number of evict entries), or <0.
 */
int64_t orc_plan(const int64_t *ids, const int64_t *iter_off, const int64_t *uniq, const int64_t *uniq_off,
                 int64_t T, int64_t total_rows, int64_t Leff, int64_t C,
                 int64_t *occ, int32_t *lookup_slots,
                 int64_t *prefetch_off, int64_t *prefetch_ids, int32_t *prefetch_slots,
                 int64_t *evict_off, int64_t *evict_ids, int32_t *evict_slots,
                 int64_t *keep_off, int64_t *keep_ids, int32_t *keep_ttl) {
    if (Leff < 1 || C < 1 || C > INT32_MAX) return ORC_ERR_ARG;
    int32_t *latest = (int32_t *)malloc((size_t)total_rows * sizeof(int32_t));
    int32_t *slot_of = (int32_t *)malloc((size_t)total_rows * sizeof(int32_t));   /* -1: not in cache */
    int32_t *ring = (int32_t *)malloc((size_t)C * sizeof(int32_t));
    if (!latest || !slot_of || !ring) { free(latest); free(slot_of); free(ring); return ORC_ERR_NOMEM; }
    for (int64_t g = 0; g < total_rows; ++g) slot_of[g] = -1;
    for (int64_t s = 0; s < C; ++s) ring[s] = (int32_t)s;
    int64_t head = 0, nfree = C;            /* ring[head .. head+nfree) mod C are the free slots, oldest first */
    int64_t pushed = 0, resident = 0, np = 0, ne = 0, nk = 0, rc = ORC_OK;
    prefetch_off[0] = evict_off[0] = keep_off[0] = 0;
    for (int64_t i = 0; i < T && rc == ORC_OK; ++i) {
        while (pushed < T && pushed - i < Leff) {
            for (int64_t k = uniq_off[pushed]; k < uniq_off[pushed + 1]; ++k) latest[uniq[k]] = (int32_t)pushed;
            ++pushed;
        }
        for (int64_t k = uniq_off[i]; k < uniq_off[i + 1]; ++k) {
            int64_t g = uniq[k];
            keep_ids[nk] = g; keep_ttl[nk] = latest[g]; ++nk;
            if (slot_of[g] < 0) {
                if (nfree == 0) { rc = ORC_ERR_CAPACITY; break; }
                int32_t s = ring[head]; head = (head + 1) % C; --nfree;
                slot_of[g] = s; ++resident;
                prefetch_ids[np] = g; prefetch_slots[np] = s; ++np;
            }
        }
        if (rc != ORC_OK) break;
        if (occ) occ[i] = resident;
        for (int64_t k = iter_off[i]; k < iter_off[i + 1]; ++k) lookup_slots[k] = slot_of[ids[k]];
        for (int64_t k = uniq_off[i]; k < uniq_off[i + 1]; ++k) {
            int64_t g = uniq[k];
            if (latest[g] == i) {
                int32_t s = slot_of[g];
                evict_ids[ne] = g; evict_slots[ne] = s; ++ne;
                ring[(head + nfree) % C] = s; ++nfree;
                slot_of[g] = -1; --resident;
            }
        }
        prefetch_off[i + 1] = np; evict_off[i + 1] = ne; keep_off[i + 1] = nk;
    }
    if (rc == ORC_OK && (resident != 0 || np != ne || nfree != C)) rc = ORC_ERR_INTERNAL;  /* cache drains */
    free(latest); free(slot_of); free(ring);
    return rc == ORC_OK ? np : rc;
}

/*
 * The plan when the lookahead may change from batch to batch (Section 4: the Oracle Cacher "can reduce" the
 * lookahead when the cache is about to fill): Algorithm 1 with the window of batch i taken as
 * [i, i + Leff_of[i] - 1].  TTL of an id of batch i = its last use inside that window, found by looking into the
 * batches of the window one by one; everything else as in orc_plan (two phases per batch, FIFO ring of free slots).
 * Same outputs as orc_plan.  Slow on purpose: O(window) per (id, batch).
 */
static int batch_has_id(const int64_t *uniq, const int64_t *uniq_off, int64_t b, int64_t g) {
    int64_t lo = uniq_off[b], hi = uniq_off[b + 1];        /* ids of a batch are sorted */
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (uniq[mid] < g) lo = mid + 1; else hi = mid;
    }
    return lo < uniq_off[b + 1] && uniq[lo] == g;
}

int64_t orc_plan_stream(const int64_t *ids, const int64_t *iter_off, const int64_t *uniq, const int64_t *uniq_off,
                        int64_t T, int64_t total_rows, const int32_t *Leff_of, int64_t C,
                        int64_t *occ, int32_t *lookup_slots,
                        int64_t *prefetch_off, int64_t *prefetch_ids, int32_t *prefetch_slots,
                        int64_t *evict_off, int64_t *evict_ids, int32_t *evict_slots,
                        int64_t *keep_off, int64_t *keep_ids, int32_t *keep_ttl) {
    if (C < 1 || C > INT32_MAX) return ORC_ERR_ARG;
    int32_t *slot_of = (int32_t *)malloc((size_t)total_rows * sizeof(int32_t));   /* -1: not in cache */
    int32_t *ring = (int32_t *)malloc((size_t)C * sizeof(int32_t));
    if (!slot_of || !ring) { free(slot_of); free(ring); return ORC_ERR_NOMEM; }
    for (int64_t g = 0; g < total_rows; ++g) slot_of[g] = -1;
    for (int64_t s = 0; s < C; ++s) ring[s] = (int32_t)s;
    int64_t head = 0, nfree = C, resident = 0, np = 0, ne = 0, nk = 0, rc = ORC_OK;
    prefetch_off[0] = evict_off[0] = keep_off[0] = 0;
    for (int64_t i = 0; i < T && rc == ORC_OK; ++i) {
        if (Leff_of[i] < 1) { rc = ORC_ERR_ARG; break; }
        int64_t last_batch = i + Leff_of[i] - 1 < T - 1 ? i + Leff_of[i] - 1 : T - 1;
        int64_t first_keep = nk;
        for (int64_t k = uniq_off[i]; k < uniq_off[i + 1]; ++k) {
            int64_t g = uniq[k];
            int64_t ttl = i;
            for (int64_t b = i + 1; b <= last_batch; ++b)
                if (batch_has_id(uniq, uniq_off, b, g)) ttl = b;
            keep_ids[nk] = g; keep_ttl[nk] = (int32_t)ttl; ++nk;
            if (slot_of[g] < 0) {
                if (nfree == 0) { rc = ORC_ERR_CAPACITY; break; }
                int32_t s = ring[head]; head = (head + 1) % C; --nfree;
                slot_of[g] = s; ++resident;
                prefetch_ids[np] = g; prefetch_slots[np] = s; ++np;
            }
        }
        if (rc != ORC_OK) break;
        if (occ) occ[i] = resident;
        for (int64_t k = iter_off[i]; k < iter_off[i + 1]; ++k) lookup_slots[k] = slot_of[ids[k]];
        for (int64_t k = first_keep; k < nk; ++k) {
            if (keep_ttl[k] == i) {
                int64_t g = keep_ids[k];
                int32_t s = slot_of[g];
                evict_ids[ne] = g; evict_slots[ne] = s; ++ne;
                ring[(head + nfree) % C] = s; ++nfree;
                slot_of[g] = -1; --resident;
            }
        }
        prefetch_off[i + 1] = np; evict_off[i + 1] = ne; keep_off[i + 1] = nk;
    }
    if (rc == ORC_OK && (resident != 0 || np != ne || nfree != C)) rc = ORC_ERR_INTERNAL;  /* cache drains */
    free(slot_of); free(ring);
    return rc == ORC_OK ? np : rc;
}

/*
 * Who uses a row (Section 3.3, logically replicated / physically partitioned caches: the Oracle Cacher marks the ids
 * that a single trainer uses, which then need no synchronisation; Section 3.3 "delayed synchronisation": of the
 * shared rows only those needed by the very next batch are synchronised on the critical path).
 * The lookups of batch i are dealt to P logical trainers by position: trainer t owns the positions
 * [cuts[i*(P+1) + t], cuts[i*(P+1) + t + 1]) counted from the batch's first lookup.
 * For every (id, batch) entry of the keep list, in its order:  owner = t when every lookup of the id in that batch is
 * trainer t's;  -1 when several trainers use it and the next batch does not;  -2 when several trainers use it and
 * the next batch uses it too.
 */
int64_t orc_keep_owners(const int64_t *ids, const int64_t *iter_off, const int64_t *uniq, const int64_t *uniq_off,
                        int64_t T, int64_t P, const int64_t *cuts, int32_t *owner) {
    if (P < 1) return ORC_ERR_ARG;
    for (int64_t i = 0; i < T; ++i) {
        const int64_t *c = cuts + i * (P + 1);
        for (int64_t q = uniq_off[i]; q < uniq_off[i + 1]; ++q) {
            int64_t g = uniq[q];
            int64_t first = -1;
            int shared = 0;
            for (int64_t k = iter_off[i]; k < iter_off[i + 1]; ++k) {
                if (ids[k] != g) continue;
                int64_t rel = k - iter_off[i], t = -1;
                for (int64_t x = 0; x < P; ++x)
                    if (rel >= c[x] && rel < c[x + 1]) t = x;
                if (t < 0) return ORC_ERR_ARG;              /* the cuts do not cover the batch */
                if (first < 0) first = t; else if (t != first) shared = 1;
            }
            int next = i + 1 < T && batch_has_id(uniq, uniq_off, i + 1, g);
            owner[q] = shared ? (next ? -2 : -1) : (int32_t)first;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ parts B and C: training */

static inline float bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16; float f; memcpy(&f, &u, 4); return f;
}
/* round-to-nearest-even fp32 -> bf16 (finite inputs; NaN kept quiet) */
static inline uint16_t f32_to_bf16(float f) {
    uint32_t u; memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static inline double load_w(const void *tab, int dtype, int64_t row, int64_t D, int64_t d) {
    return dtype == ORC_F32 ? (double)((const float *)tab)[row * D + d]
                            : (double)bf16_to_f32(((const uint16_t *)tab)[row * D + d]);
}
/* fp64 -> storage type; for bf16 the value is first rounded to fp32 (the arithmetic type of the path) */
static inline void store_w(void *tab, int dtype, int64_t row, int64_t D, int64_t d, double v) {
    if (dtype == ORC_F32) ((float *)tab)[row * D + d] = (float)v;
    else ((uint16_t *)tab)[row * D + d] = f32_to_bf16((float)v);
}

/*
 * Optimizer step on one row, fp32 storage: the plain rules in fp64, each stored value rounded once.
 * G[d] is the fp64 sum of the row's gradients.
 */
static int update_row_f64(float *table, float *state, int64_t row, int64_t D, int optimizer, float lr, float eps,
                          const double *G) {
    const double lrd = (double)lr, epsd = (double)eps;
    float *w = table + row * D;
    if (optimizer == ORC_SGD) {
        for (int64_t d = 0; d < D; ++d) w[d] = (float)((double)w[d] - lrd * G[d]);
    } else if (optimizer == ORC_ADAGRAD) {
        for (int64_t d = 0; d < D; ++d) {
            float s = (float)((double)state[row * D + d] + G[d] * G[d]);
            state[row * D + d] = s;
            w[d] = (float)((double)w[d] - lrd * G[d] / (sqrt((double)s) + epsd));
        }
    } else if (optimizer == ORC_ADAGRAD_ROWWISE) {
        double ms = 0.0;
        for (int64_t d = 0; d < D; ++d) ms += G[d] * G[d];
        float s = (float)((double)state[row] + ms / (double)D);
        state[row] = s;
        double den = sqrt((double)s) + epsd;
        for (int64_t d = 0; d < D; ++d) w[d] = (float)((double)w[d] - lrd * G[d] / den);
    } else return ORC_ERR_ARG;
    return ORC_OK;
}

/*
 * Optimizer step on one row, bf16 storage.  The stored value is a quantised code, so the value that gets
 * rounded to bf16 must be formed in the arithmetic type the workload fixes for this case, fp32
 * ("bf16 storage, fp32 accumulation / optimizer"): sums (the gradient sum, the row-wise mean of squares)
 * are taken in fp64 and rounded once to fp32, which makes them independent of the order of addition;
 * every element-wise operation is one correctly rounded fp32 operation, written out one per line.
 */
static int update_row_bf16(uint16_t *table, float *state, int64_t row, int64_t D, int optimizer, float lr,
                           float eps, const double *G) {
    uint16_t *w = table + row * D;
    float den_row = 0.0f;
    if (optimizer == ORC_ADAGRAD_ROWWISE) {
        double ms = 0.0;
        for (int64_t d = 0; d < D; ++d) { float g = (float)G[d]; ms += (double)g * (double)g; }
        float mean = (float)(ms / (double)D);
        float s = state[row] + mean;
        state[row] = s;
        den_row = sqrtf(s) + eps;
    } else if (optimizer != ORC_SGD && optimizer != ORC_ADAGRAD) return ORC_ERR_ARG;
    for (int64_t d = 0; d < D; ++d) {
        float g = (float)G[d];
        float wv = bf16_to_f32(w[d]);
        float step = lr * g;
        if (optimizer == ORC_ADAGRAD) {
            float gg = g * g;
            float s = state[row * D + d] + gg;
            state[row * D + d] = s;
            float den = sqrtf(s) + eps;
            step = step / den;
        } else if (optimizer == ORC_ADAGRAD_ROWWISE) {
            step = step / den_row;
        }
        float wn = wv - step;
        w[d] = f32_to_bf16(wn);
    }
    return ORC_OK;
}

typedef struct { int64_t row; int64_t pos; } rowpos_t;
static int cmp_rowpos(const void *a, const void *b) {
    const rowpos_t *x = (const rowpos_t *)a, *y = (const rowpos_t *)b;
    if (x->row != y->row) return (x->row > y->row) - (x->row < y->row);
    return (x->pos > y->pos) - (x->pos < y->pos);
}

/* forward of the bags [b0, b1): out[bag, :] = sum of the bag's rows in lookup order, fp64, rounded once */
static void forward_bags(const void *table, int dtype, int64_t D, const int64_t *row_idx, const int64_t *bag_off,
                         int64_t b0, int64_t b1, float *out) {
    for (int64_t b = b0; b < b1; ++b)
        for (int64_t d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int64_t k = bag_off[b]; k < bag_off[b + 1]; ++k) acc += load_w(table, dtype, row_idx[k], D, d);
            out[b * D + d] = (float)acc;
        }
}

/*
 * backward + update for the lookups listed in rp[0 .. m), sorted by (row, position): for every distinct row the
 * gradient rows of its lookups are added in ascending position (fp64), then the row is updated once.
 * G is scratch for D doubles.
 */
static int update_sorted_rows(void *table, float *state, int64_t D, int dtype, int optimizer, float lr, float eps,
                              const rowpos_t *rp, int64_t m, const int64_t *bag_of, const float *grad_out, double *G) {
    for (int64_t a = 0; a < m;) {
        int64_t b = a, row = rp[a].row;
        for (int64_t d = 0; d < D; ++d) G[d] = 0.0;
        for (; b < m && rp[b].row == row; ++b) {
            const float *g = grad_out + bag_of[rp[b].pos] * D;
            for (int64_t d = 0; d < D; ++d) G[d] += (double)g[d];
        }
        int rc = dtype == ORC_F32 ? update_row_f64((float *)table, state, row, D, optimizer, lr, eps, G)
                                  : update_row_bf16((uint16_t *)table, state, row, D, optimizer, lr, eps, G);
        if (rc != ORC_OK) return rc;
        a = b;
    }
    return ORC_OK;
}

/*
 * One training iteration on `table` (the full table with rows = global ids, or the cache with
 * rows = slots):
 *   forward   out[bag, :] = sum over the bag's lookups of table[row, :]   (lookup order; empty bag = 0)
 *   backward  G[row, :]   = sum of grad_out[bag(k), :] over the lookups k of that row, ascending k
 *   update    once per distinct row:
 *               SGD               w -= lr * G
 *               Adagrad           s += G*G (per element);        w -= lr * G / (sqrt(s) + eps)
 *               row-wise Adagrad  s_row += mean_d(G_d^2);        w -= lr * G / (sqrt(s_row) + eps)
 * state: fp32 [rows][D] (Adagrad), fp32 [rows] (row-wise), unused (SGD).  The forward uses the weights
 * before the update.  out may be NULL (skip forward); grad_out may be NULL (skip backward+update).
 */
int orc_train_iter(void *table, float *state, int64_t rows, int64_t D, int dtype, int optimizer, float lr,
                   float eps, const int64_t *row_idx, int64_t n, const int64_t *bag_off, int64_t bags,
                   const float *grad_out, float *out) {
    if (bag_off[0] != 0 || bag_off[bags] != n) return ORC_ERR_ARG;
    for (int64_t k = 0; k < n; ++k) if (row_idx[k] < 0 || row_idx[k] >= rows) return ORC_ERR_ID_RANGE;
    if (out) forward_bags(table, dtype, D, row_idx, bag_off, 0, bags, out);
    if (!grad_out || n == 0) return ORC_OK;
    rowpos_t *rp = (rowpos_t *)malloc((size_t)n * sizeof(rowpos_t));
    int64_t *bag_of = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    double *G = (double *)malloc((size_t)D * sizeof(double));
    if (!rp || !bag_of || !G) { free(rp); free(bag_of); free(G); return ORC_ERR_NOMEM; }
    for (int64_t b = 0; b < bags; ++b)
        for (int64_t k = bag_off[b]; k < bag_off[b + 1]; ++k) bag_of[k] = b;
    for (int64_t k = 0; k < n; ++k) { rp[k].row = row_idx[k]; rp[k].pos = k; }
    qsort(rp, (size_t)n, sizeof(rowpos_t), cmp_rowpos);
    int rc = update_sorted_rows(table, state, D, dtype, optimizer, lr, eps, rp, n, bag_of, grad_out, G);
    free(rp); free(bag_of); free(G);
    return rc;
}

/*
 * The same iteration on several host threads, for tables and traces at the full sizes of the workloads.  Nothing
 * about the arithmetic changes: a bag is still summed by one thread in lookup order, and a row's gradients are
 * still added by one thread in ascending position and the row updated once, so the result equals orc_train_iter's
 * bit for bit (tests compare them).  Thread t takes the bags [t*bags/P, (t+1)*bags/P) in the forward, and the rows
 * with row % P == t in the backward (it picks its lookups out of the batch in ascending position and sorts them by
 * row); the forward of all threads ends before any update starts.
 */
typedef struct {
    void *table; float *state; int64_t D; int dtype, optimizer; float lr, eps;
    const int64_t *row_idx; int64_t n; const int64_t *bag_off; int64_t bags;
    const float *grad_out; float *out; const int64_t *bag_of;
    int t, P, phase, rc;
} mt_job_t;

static void *mt_worker(void *arg) {
    mt_job_t *j = (mt_job_t *)arg;
    j->rc = ORC_OK;
    if (j->phase == 0) {
        forward_bags(j->table, j->dtype, j->D, j->row_idx, j->bag_off, j->bags * j->t / j->P,
                     j->bags * (j->t + 1) / j->P, j->out);
        return NULL;
    }
    int64_t m = 0;
    for (int64_t k = 0; k < j->n; ++k) m += (j->row_idx[k] % j->P) == j->t;
    rowpos_t *rp = (rowpos_t *)malloc((size_t)(m > 0 ? m : 1) * sizeof(rowpos_t));
    double *G = (double *)malloc((size_t)j->D * sizeof(double));
    if (!rp || !G) { free(rp); free(G); j->rc = ORC_ERR_NOMEM; return NULL; }
    int64_t w = 0;
    for (int64_t k = 0; k < j->n; ++k)
        if ((j->row_idx[k] % j->P) == j->t) { rp[w].row = j->row_idx[k]; rp[w].pos = k; ++w; }
    qsort(rp, (size_t)m, sizeof(rowpos_t), cmp_rowpos);
    j->rc = update_sorted_rows(j->table, j->state, j->D, j->dtype, j->optimizer, j->lr, j->eps, rp, m, j->bag_of,
                               j->grad_out, G);
    free(rp); free(G);
    return NULL;
}

int orc_train_iter_mt(void *table, float *state, int64_t rows, int64_t D, int dtype, int optimizer, float lr,
                      float eps, const int64_t *row_idx, int64_t n, const int64_t *bag_off, int64_t bags,
                      const float *grad_out, float *out, int threads) {
    if (threads < 1 || threads > 256) return ORC_ERR_ARG;
    if (bag_off[0] != 0 || bag_off[bags] != n) return ORC_ERR_ARG;
    if (optimizer != ORC_SGD && optimizer != ORC_ADAGRAD && optimizer != ORC_ADAGRAD_ROWWISE) return ORC_ERR_ARG;
    for (int64_t k = 0; k < n; ++k) if (row_idx[k] < 0 || row_idx[k] >= rows) return ORC_ERR_ID_RANGE;
    int64_t *bag_of = NULL;
    if (grad_out && n > 0) {
        bag_of = (int64_t *)malloc((size_t)n * sizeof(int64_t));
        if (!bag_of) return ORC_ERR_NOMEM;
        for (int64_t b = 0; b < bags; ++b)
            for (int64_t k = bag_off[b]; k < bag_off[b + 1]; ++k) bag_of[k] = b;
    }
    mt_job_t *jobs = (mt_job_t *)malloc((size_t)threads * sizeof(mt_job_t));
    pthread_t *tid = (pthread_t *)malloc((size_t)threads * sizeof(pthread_t));
    if (!jobs || !tid) { free(jobs); free(tid); free(bag_of); return ORC_ERR_NOMEM; }
    int rc = ORC_OK;
    for (int phase = 0; phase < 2 && rc == ORC_OK; ++phase) {
        if (phase == 0 && !out) continue;
        if (phase == 1 && !bag_of) continue;
        int started = 0;
        for (int t = 0; t < threads; ++t) {
            mt_job_t j = {table, state, D, dtype, optimizer, lr, eps, row_idx, n, bag_off, bags, grad_out, out, bag_of,
                          t, threads, phase, ORC_OK};
            jobs[t] = j;
            if (pthread_create(&tid[t], NULL, mt_worker, &jobs[t]) != 0) { rc = ORC_ERR_INTERNAL; break; }
            ++started;
        }
        for (int t = 0; t < started; ++t) {
            pthread_join(tid[t], NULL);
            if (jobs[t].rc != ORC_OK && rc == ORC_OK) rc = jobs[t].rc;
        }
    }
    free(jobs); free(tid); free(bag_of);
    return rc;
}

/*
 * Cache maintenance between iterations (the trainer-side duties of Section 3.4 "Trainer"): first write
 * every evicted row (weights and optimizer state) back to the full table, then load every prefetched
 * row into its slot.  Rows are copied bit for bit.
 */
int orc_cache_apply(void *cache_w, float *cache_state, void *host_w, float *host_state, int64_t C, int64_t rows,
                    int64_t D, int dtype, int optimizer,
                    const int64_t *evict_ids, const int32_t *evict_slots, int64_t n_evict,
                    const int64_t *prefetch_ids, const int32_t *prefetch_slots, int64_t n_prefetch) {
    size_t rb = (size_t)D * (dtype == ORC_F32 ? 4 : 2);
    size_t sb = optimizer == ORC_ADAGRAD ? (size_t)D * 4 : optimizer == ORC_ADAGRAD_ROWWISE ? 4 : 0;
    for (int pass = 0; pass < 2; ++pass) {
        const int64_t *gi = pass == 0 ? evict_ids : prefetch_ids;
        const int32_t *si = pass == 0 ? evict_slots : prefetch_slots;
        int64_t cnt = pass == 0 ? n_evict : n_prefetch;
        for (int64_t k = 0; k < cnt; ++k) {
            if (gi[k] < 0 || gi[k] >= rows || si[k] < 0 || si[k] >= C) return ORC_ERR_ID_RANGE;
            char *h = (char *)host_w + (size_t)gi[k] * rb, *c = (char *)cache_w + (size_t)si[k] * rb;
            if (pass == 0) memcpy(h, c, rb); else memcpy(c, h, rb);
            if (sb) {
                char *hs = (char *)host_state + (size_t)gi[k] * sb, *cs = (char *)cache_state + (size_t)si[k] * sb;
                if (pass == 0) memcpy(hs, cs, sb); else memcpy(cs, hs, sb);
            }
        }
    }
    return ORC_OK;
}
