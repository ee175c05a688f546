/*
 * CPU oracle for the GPUVM hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, sequential, deliberately slow C.  It shares no code, header, table or
 * helper with the HIP library and must never be linked into, imported by or
 * called from the product path; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg use it.
 *
 * Part 1 - the application computed directly on host memory.  GPUVM's paging
 *   is transparent: a kernel indexing a gpuvm<T> array computes what the same
 *   kernel computes on ordinary memory (paper, System Overview, the
 *   vector-addition listing).  So the expected output of every workload is its
 *   plain definition, written out here with no paging at all.
 *
 * Part 2 - a sequential simulator of the paged memory (paper, "Paged Memory
 *   System Design": page mapping, eviction scheme, page access
 *   synchronization; "Oversubscription Analysis": FIFO-based reference
 *   priority eviction).  It takes the steps in the paper's order: look the
 *   page up, count the group of accessors as users (reference counter), for a
 *   missing page draw the next frame from the circular buffer's global head
 *   cursor, never reuse a frame whose reference counter is non-zero, evict
 *   the page that lives there (write it to the host), establish the new
 *   mapping, then let the accessors proceed.
 *
 *   Readings of points the paper leaves open (also listed in the design notes):
 *     - a frame whose counter is non-zero is passed over (next cursor
 *       position) rather than waited for;
 *     - the CLOCK policy adds a reference bit, set when a page is installed
 *       and whenever it is used, cleared when the cursor passes; FIFO is the
 *       same walk without that test;
 *     - a victim is written back only if it was written to (dirty bit);
 *     - the write-aware CLOCK variant (the paper only names the idea: delay
 *       the eviction of write-intensive pages) passes over a dirty page once
 *       more after its reference bit is clear, then evicts it;
 *     - the generalized CLOCK variant (not in the paper; the classical GCLOCK
 *       with a small counter) keeps a use count of 0..2 instead of the bit:
 *       installed at 0, raised by every later use, lowered by the passing
 *       cursor, evicted at 0 - pages earn their chances by being used again,
 *       and a scan never makes the cursor pass anything;
 *     - two hands (optional, the CLOCK policies only; the classical two-handed
 *       clock of 4.2BSD, not in the paper): with a spread of S > 0 positions a
 *       front hand runs S frames ahead of the cursor and clears the reference
 *       bit of the frame it stands on, every time the cursor advances; the
 *       cursor itself then passes a frame only if its page was used again
 *       after the front hand went by (and clears the bit, as before).  A page
 *       keeps its first bit from its installation until the front hand reaches
 *       it, so fresh pages are safe for F - S positions, and a page that is
 *       never used again is taken at the cursor's first visit: a scan makes
 *       the cursor pass nothing.  S = 0 is the one-handed CLOCK above;
 *     - accesses arrive in phases (a group of accesses that are in flight
 *       together); each distinct page of a phase counts one hit or one fault;
 *       its faults are served in ascending page order; pins are dropped when
 *       the phase ends.  A phase of one access gives the textbook policies.
 *
 * Parity pins: see tests/test_oracle_*.py (textbook fault counts, closed
 * forms, brute force against independently written models, invariants).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Part 1: applications on plain host memory                           */
/* ------------------------------------------------------------------ */

/* Random gather: out[k] = host[idx[k]], sum = sum_k out[k] (64-bit). */
void oracle_gather(const uint32_t *host, const uint32_t *idx, uint64_t n,
                   uint32_t *out, uint64_t *sum)
{
    uint64_t s = 0;
    for (uint64_t k = 0; k < n; ++k) {
        out[k] = host[idx[k]];
        s += (uint64_t)out[k];
    }
    *sum = s;
}

/* Vector addition (the paper's listing): c[i] = a[i] + b[i], one fp32 rounding. */
void oracle_vector_add(const float *a, const float *b, float *c, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) {
        volatile float s = a[i] + b[i];
        c[i] = s;
    }
}

/* Streaming read-reduce: for every pass and every block of block_elems
 * consecutive floats, the double-precision sum taken in index order.
 * s is laid out [pass][block]; the last block may be short. */
void oracle_stream_reduce(const float *x, uint64_t n, uint64_t block_elems,
                          int passes, double *s)
{
    uint64_t nblocks = (n + block_elems - 1) / block_elems;
    for (int p = 0; p < passes; ++p) {
        for (uint64_t b = 0; b < nblocks; ++b) {
            uint64_t lo = b * block_elems;
            uint64_t hi = lo + block_elems < n ? lo + block_elems : n;
            double acc = 0.0;
            for (uint64_t i = lo; i < hi; ++i) acc += (double)x[i];
            s[(uint64_t)p * nblocks + b] = acc;
        }
    }
}

/* Sum of |x| per block (the scale the fp tolerance is relative to). */
void oracle_stream_abs(const float *x, uint64_t n, uint64_t block_elems, double *s)
{
    uint64_t nblocks = (n + block_elems - 1) / block_elems;
    for (uint64_t b = 0; b < nblocks; ++b) {
        uint64_t lo = b * block_elems;
        uint64_t hi = lo + block_elems < n ? lo + block_elems : n;
        double acc = 0.0;
        for (uint64_t i = lo; i < hi; ++i) acc += x[i] < 0 ? -(double)x[i] : (double)x[i];
        s[b] = acc;
    }
}

/* Breadth-first search from src on a directed CSR graph: level[v] = number of
 * hops of a shortest path, -1 when v cannot be reached.  Queue BFS.
 * Returns 0, or -1 if the queue could not be allocated. */
int oracle_bfs(const int64_t *row_ptr, const int32_t *col_idx, int64_t nv,
               int64_t src, int32_t *level)
{
    int32_t *queue = (int32_t *)malloc((size_t)nv * sizeof(int32_t));
    if (!queue) return -1;
    for (int64_t v = 0; v < nv; ++v) level[v] = -1;
    int64_t head = 0, tail = 0;
    level[src] = 0;
    queue[tail++] = (int32_t)src;
    while (head < tail) {
        int32_t u = queue[head++];
        for (int64_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) {
            int32_t v = col_idx[e];
            if (level[v] < 0) {
                level[v] = level[u] + 1;
                queue[tail++] = v;
            }
        }
    }
    free(queue);
    return 0;
}

/* Weakly connected components: label[v] = smallest vertex id in v's component
 * when edge directions are ignored.  Plain label propagation to the fixed
 * point: sweep all edges, pull both ends down to the smaller label, repeat
 * until a sweep changes nothing.  Returns the number of sweeps. */
int oracle_cc(const int64_t *row_ptr, const int32_t *col_idx, int64_t nv, int32_t *label)
{
    for (int64_t v = 0; v < nv; ++v) label[v] = (int32_t)v;
    int sweeps = 0, changed = 1;
    while (changed) {
        changed = 0;
        ++sweeps;
        for (int64_t v = 0; v < nv; ++v)
            for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                int32_t u = col_idx[e];
                if (label[v] < label[u]) { label[u] = label[v]; changed = 1; }
                else if (label[u] < label[v]) { label[v] = label[u]; changed = 1; }
            }
    }
    return sweeps;
}

/* Single-source shortest paths with non-negative integer weights, Bellman-Ford:
 * relax every edge until a full sweep changes nothing.  dist[v] = 0xFFFFFFFF
 * when v cannot be reached.  Returns the number of sweeps. */
int oracle_sssp(const int64_t *row_ptr, const int32_t *col_idx, const uint32_t *weight,
                int64_t nv, int64_t src, uint32_t *dist)
{
    for (int64_t v = 0; v < nv; ++v) dist[v] = 0xFFFFFFFFu;
    dist[src] = 0;
    int sweeps = 0, changed = 1;
    while (changed) {
        changed = 0;
        ++sweeps;
        for (int64_t v = 0; v < nv; ++v) {
            if (dist[v] == 0xFFFFFFFFu) continue;
            for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                uint64_t nd = (uint64_t)dist[v] + weight[e];
                if (nd < dist[col_idx[e]]) { dist[col_idx[e]] = (uint32_t)nd; changed = 1; }
            }
        }
    }
    return sweeps;
}

/* Embedding bag, sum pooling: out[bag][c] = sum_j table[ids[bag][j]][c].
 * Accumulated in double precision (the definition of the sum). */
void oracle_embedding_bag(const float *table, uint64_t dim, const int32_t *ids,
                          uint64_t bags, uint64_t bag_len, double *out)
{
    for (uint64_t b = 0; b < bags; ++b)
        for (uint64_t c = 0; c < dim; ++c) {
            double acc = 0.0;
            for (uint64_t j = 0; j < bag_len; ++j)
                acc += (double)table[(uint64_t)ids[b * bag_len + j] * dim + c];
            out[b * dim + c] = acc;
        }
}

/* Same sum taken the way the workload states it: fp32 output, the bag's rows
 * added one after the other in the order they are listed, in fp32. */
void oracle_embedding_bag_f32(const float *table, uint64_t dim, const int32_t *ids,
                              uint64_t bags, uint64_t bag_len, float *out)
{
    for (uint64_t b = 0; b < bags; ++b)
        for (uint64_t c = 0; c < dim; ++c) {
            volatile float acc = 0.0f;      /* volatile: one rounding per add */
            for (uint64_t j = 0; j < bag_len; ++j)
                acc = acc + table[(uint64_t)ids[b * bag_len + j] * dim + c];
            out[b * dim + c] = acc;
        }
}

/* Sum of |.| per output element of the bag (tolerance scale). */
void oracle_embedding_bag_abs(const float *table, uint64_t dim, const int32_t *ids,
                              uint64_t bags, uint64_t bag_len, double *out)
{
    for (uint64_t b = 0; b < bags; ++b)
        for (uint64_t c = 0; c < dim; ++c) {
            double acc = 0.0;
            for (uint64_t j = 0; j < bag_len; ++j) {
                double t = (double)table[(uint64_t)ids[b * bag_len + j] * dim + c];
                acc += t < 0 ? -t : t;
            }
            out[b * dim + c] = acc;
        }
}

/* Matrix-vector product: y[i] = sum_j A[i][j] * x[j], row-major A, double
 * precision, j ascending (the row-per-thread kernel of the paper's
 * transfer-bound applications: MVT's first product, ATAX's first step);
 * yabs[i] = sum_j |A[i][j] * x[j]| (tolerance scale). */
void oracle_matvec(const float *A, uint64_t rows, uint64_t cols, const float *x,
                   double *y, double *yabs)
{
    for (uint64_t i = 0; i < rows; ++i) {
        double acc = 0.0, aabs = 0.0;
        for (uint64_t j = 0; j < cols; ++j) {
            double t = (double)A[i * cols + j] * (double)x[j];
            acc += t;
            aabs += t < 0 ? -t : t;
        }
        y[i] = acc;
        if (yabs) yabs[i] = aabs;
    }
}

/* Transposed matrix-vector product: y[j] = sum_i A[i][j] * x[i], row-major A,
 * double precision; yabs[j] = sum_i |A[i][j] * x[i]| (tolerance scale). */
void oracle_matvec_t(const float *A, uint64_t rows, uint64_t cols, const float *x,
                     double *y, double *yabs)
{
    for (uint64_t j = 0; j < cols; ++j) {
        double acc = 0.0, aabs = 0.0;
        for (uint64_t i = 0; i < rows; ++i) {
            double t = (double)A[i * cols + j] * (double)x[i];
            acc += t;
            aabs += t < 0 ? -t : t;
        }
        y[j] = acc;
        if (yabs) yabs[j] = aabs;
    }
}

/* Filter then gather: count the rows with key > threshold and sum val over them. */
void oracle_filter_sum(const uint32_t *key, const uint32_t *val, uint64_t n,
                       uint32_t threshold, uint64_t *count, uint64_t *sum)
{
    uint64_t c = 0, s = 0;
    for (uint64_t i = 0; i < n; ++i)
        if (key[i] > threshold) { c += 1; s += val[i]; }
    *count = c;
    *sum = s;
}

/* Scatter-increment: host[idx[k]] += 1 for every k. */
void oracle_scatter_increment(uint64_t *host, const uint32_t *idx, uint64_t k)
{
    for (uint64_t i = 0; i < k; ++i) host[idx[i]] += 1;
}

/* ------------------------------------------------------------------ */
/* Part 2: sequential paged-memory simulator                           */
/* ------------------------------------------------------------------ */

enum { SIM_FIFO = 0, SIM_CLOCK = 1, SIM_CLOCK_WA = 3, SIM_GCLOCK = 4 };   /* 2 (wait for the drawn frame) has no sequential meaning */

/* SIM_GCLOCK: generalized CLOCK with a use count of 0..2 per frame, kept in the
 * two flag bytes ref (count >= 1) and defer (count == 2).  A page is installed
 * with count 0, every later use raises the count by one up to 2, the hand
 * lowers a positive count by one and passes, and takes a frame at count 0. */
static void sim_mark_used(uint8_t *ref, uint8_t *defer, int policy)
{
    if (policy == SIM_GCLOCK && *ref) *defer = 1;
    *ref = 1;
}
enum { SIM_READ = 0, SIM_WRITE = 1, SIM_ADD = 2 };
enum {
    SIM_C_FAULTS = 0, SIM_C_HITS, SIM_C_EVICTIONS, SIM_C_WB_EVICT,
    SIM_C_WB_FLUSH, SIM_C_SKIPS, SIM_C_SWEEPS, SIM_C_PHASES, SIM_NCOUNTERS
};

typedef struct sim {
    uint64_t *host;        /* backing store in 8-byte words, may be NULL   */
    uint64_t n_words, page_words, n_pages, n_frames;
    int policy;
    int64_t *owner;        /* per frame: page living there, -1 = empty     */
    uint8_t *ref, *dirty;  /* per frame                                    */
    uint8_t *defer;        /* per frame: dirty page already spared once    */
    uint32_t *pin;         /* per frame: reference counter                 */
    int64_t *where;        /* per page: frame, -1 = not in GPU memory      */
    uint64_t *frames;      /* n_frames x page_words when host != NULL      */
    uint64_t hand;         /* global head cursor of the circular buffer    */
    uint64_t spread;       /* two-handed CLOCK: front hand this far ahead, 0 = one hand */
    uint64_t counters[SIM_NCOUNTERS];
    uint8_t *seen;         /* per page scratch: member of current phase    */
} sim_t;

void sim_destroy(sim_t *s)
{
    if (!s) return;
    free(s->owner); free(s->ref); free(s->dirty); free(s->pin); free(s->defer);
    free(s->where); free(s->frames); free(s->seen); free(s);
}

sim_t *sim_create(uint64_t *host, uint64_t n_words, uint64_t page_words,
                  uint64_t n_frames, int policy)
{
    if (page_words == 0 || n_frames == 0 || n_words == 0) return NULL;
    sim_t *s = (sim_t *)calloc(1, sizeof(sim_t));
    if (!s) return NULL;
    s->host = host; s->n_words = n_words; s->page_words = page_words;
    s->n_pages = (n_words + page_words - 1) / page_words;
    s->n_frames = n_frames; s->policy = policy;
    s->owner = (int64_t *)malloc(n_frames * sizeof(int64_t));
    s->ref = (uint8_t *)calloc(n_frames, 1);
    s->dirty = (uint8_t *)calloc(n_frames, 1);
    s->defer = (uint8_t *)calloc(n_frames, 1);
    s->pin = (uint32_t *)calloc(n_frames, sizeof(uint32_t));
    s->where = (int64_t *)malloc(s->n_pages * sizeof(int64_t));
    s->seen = (uint8_t *)calloc(s->n_pages, 1);
    s->frames = host ? (uint64_t *)calloc(n_frames * page_words, 8) : NULL;
    if (policy != SIM_FIFO && policy != SIM_CLOCK && policy != SIM_CLOCK_WA && policy != SIM_GCLOCK) { sim_destroy(s); return NULL; }
    if (!s->owner || !s->ref || !s->dirty || !s->defer || !s->pin || !s->where || !s->seen ||
        (host && !s->frames)) { sim_destroy(s); return NULL; }
    for (uint64_t f = 0; f < n_frames; ++f) s->owner[f] = -1;
    for (uint64_t p = 0; p < s->n_pages; ++p) s->where[p] = -1;
    return s;
}

static uint64_t page_len(const sim_t *s, uint64_t page)
{
    uint64_t lo = page * s->page_words;
    return lo + s->page_words <= s->n_words ? s->page_words : s->n_words - lo;
}

static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return x < y ? -1 : x > y;
}

/* Serve one page fault: walk the circular buffer from the head cursor until a
 * frame may be taken, evict what lives there, install page p pinned once. */
static void sim_fault(sim_t *s, uint64_t p)
{
    uint64_t f;
    s->counters[SIM_C_FAULTS]++;
    for (;;) {
        f = s->hand;
        s->hand = (s->hand + 1) % s->n_frames;
        if (s->spread && (s->policy == SIM_CLOCK || s->policy == SIM_CLOCK_WA)) {
            /* the front hand moves with the cursor and clears the bit it stands on */
            uint64_t g = (f + s->spread) % s->n_frames;
            if (g != f && s->owner[g] >= 0) s->ref[g] = 0;
        }
        if (s->owner[f] < 0) break;                       /* never used yet */
        if (s->pin[f] > 0) { s->counters[SIM_C_SKIPS]++; continue; }
        if ((s->policy == SIM_CLOCK || s->policy == SIM_CLOCK_WA) && s->ref[f]) {
            s->ref[f] = 0; s->counters[SIM_C_SWEEPS]++; continue;
        }
        if (s->policy == SIM_CLOCK_WA && s->dirty[f] && !s->defer[f]) {
            s->defer[f] = 1; s->counters[SIM_C_SWEEPS]++; continue;   /* spare a written page once */
        }
        if (s->policy == SIM_GCLOCK && (s->defer[f] || s->ref[f])) {  /* count 2 -> 1 -> 0 */
            if (s->defer[f]) s->defer[f] = 0; else s->ref[f] = 0;
            s->counters[SIM_C_SWEEPS]++; continue;
        }
        uint64_t q = (uint64_t)s->owner[f];
        s->counters[SIM_C_EVICTIONS]++;
        if (s->dirty[f]) {
            s->counters[SIM_C_WB_EVICT]++;
            if (s->host)
                memcpy(s->host + q * s->page_words, s->frames + f * s->page_words,
                       page_len(s, q) * 8);
        }
        s->where[q] = -1;
        break;
    }
    s->owner[f] = (int64_t)p;
    s->where[p] = (int64_t)f;
    s->dirty[f] = 0; s->defer[f] = 0; s->ref[f] = s->policy == SIM_GCLOCK ? 0 : 1; s->pin[f] = 1;
    if (s->host)
        memcpy(s->frames + f * s->page_words, s->host + p * s->page_words,
               page_len(s, p) * 8);
}

/* One phase of k accesses that are in flight together.
 * word_idx[i]: 8-byte word touched; op[i]: SIM_READ / SIM_WRITE / SIM_ADD;
 * val[i]: operand of WRITE / ADD (may be NULL if every op is READ);
 * out[i]: word value seen by a READ, value before the update for ADD (may be
 * NULL; needs a backing store).
 * Returns 0; -1 index out of range; -2 more distinct pages than frames. */
int sim_phase(sim_t *s, const uint64_t *word_idx, const uint8_t *op,
              const uint64_t *val, uint64_t k, uint64_t *out)
{
    uint64_t *pages = (uint64_t *)malloc((k ? k : 1) * sizeof(uint64_t));
    uint64_t nu = 0;
    if (!pages) return -3;
    for (uint64_t i = 0; i < k; ++i) {
        if (word_idx[i] >= s->n_words) { free(pages); return -1; }
        uint64_t p = word_idx[i] / s->page_words;
        if (!s->seen[p]) { s->seen[p] = 1; pages[nu++] = p; }
    }
    for (uint64_t i = 0; i < nu; ++i) s->seen[pages[i]] = 0;
    if (nu > s->n_frames) { free(pages); return -2; }
    s->counters[SIM_C_PHASES]++;
    qsort(pages, nu, sizeof(uint64_t), cmp_u64);
    /* pages already in GPU memory: one more user each, marked as used */
    for (uint64_t i = 0; i < nu; ++i) {
        int64_t f = s->where[pages[i]];
        if (f >= 0) { s->pin[f]++; sim_mark_used(&s->ref[f], &s->defer[f], s->policy); s->counters[SIM_C_HITS]++; s->seen[pages[i]] = 2; }
    }
    /* missing pages, ascending */
    for (uint64_t i = 0; i < nu; ++i) {
        if (s->seen[pages[i]] == 2) { s->seen[pages[i]] = 0; continue; }
        sim_fault(s, pages[i]);
    }
    /* the accesses themselves, in index order */
    for (uint64_t i = 0; i < k; ++i) {
        uint64_t p = word_idx[i] / s->page_words, o = word_idx[i] % s->page_words;
        uint64_t f = (uint64_t)s->where[p];
        uint64_t *w = s->frames ? s->frames + f * s->page_words + o : NULL;
        if (op[i] == SIM_READ) {
            if (w && out) out[i] = *w;
        } else {
            s->dirty[f] = 1;
            if (w) {
                if (out) out[i] = *w;
                *w = (op[i] == SIM_WRITE) ? val[i] : *w + val[i];
            }
        }
    }
    for (uint64_t i = 0; i < nu; ++i) s->pin[s->where[pages[i]]]--;
    free(pages);
    return 0;
}

/* n accesses cut into phases of phase_len consecutive accesses. */
int sim_run(sim_t *s, const uint64_t *word_idx, const uint8_t *op,
            const uint64_t *val, uint64_t n, uint64_t phase_len, uint64_t *out)
{
    for (uint64_t lo = 0; lo < n; lo += phase_len) {
        uint64_t k = lo + phase_len <= n ? phase_len : n - lo;
        int rc = sim_phase(s, word_idx + lo, op + lo, val ? val + lo : NULL, k,
                           out ? out + lo : NULL);
        if (rc) return rc;
    }
    return 0;
}

/* Write every dirty page back to the host; pages stay mapped, clean. */
void sim_flush(sim_t *s)
{
    for (uint64_t f = 0; f < s->n_frames; ++f) {
        if (s->owner[f] >= 0 && s->dirty[f]) {
            uint64_t q = (uint64_t)s->owner[f];
            s->counters[SIM_C_WB_FLUSH]++;
            if (s->host)
                memcpy(s->host + q * s->page_words, s->frames + f * s->page_words,
                       page_len(s, q) * 8);
            s->dirty[f] = 0;
            if (s->policy != SIM_GCLOCK) s->defer[f] = 0;   /* there it is half of the use count */
        }
    }
}

/* Two-handed CLOCK: distance of the front hand from the cursor, in frames
 * (0 = one hand; taken modulo the number of frames).  Returns 0, or -1 for a
 * policy without a reference bit. */
int sim_set_spread(sim_t *s, uint64_t spread)
{
    if (spread && s->policy != SIM_CLOCK && s->policy != SIM_CLOCK_WA) return -1;
    s->spread = spread % s->n_frames;
    return 0;
}

void sim_counters(const sim_t *s, uint64_t *out)
{
    memcpy(out, s->counters, sizeof(s->counters));
}

uint64_t sim_hand(const sim_t *s) { return s->hand; }

/* owner/ref/dirty/pin per frame, where per page (any pointer may be NULL). */
void sim_state(const sim_t *s, int64_t *owner, uint8_t *ref, uint8_t *dirty,
               uint32_t *pin, int64_t *where, uint8_t *defer)
{
    if (defer) memcpy(defer, s->defer, s->n_frames);
    if (owner) memcpy(owner, s->owner, s->n_frames * sizeof(int64_t));
    if (ref)   memcpy(ref, s->ref, s->n_frames);
    if (dirty) memcpy(dirty, s->dirty, s->n_frames);
    if (pin)   memcpy(pin, s->pin, s->n_frames * sizeof(uint32_t));
    if (where) memcpy(where, s->where, s->n_pages * sizeof(int64_t));
}
