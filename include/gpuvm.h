/*
 * gpuvm.h - host-side C ABI of libgpuvm: GPU-driven demand paging for MI355X.
 *
 * GPU threads, not the CPU or the OS, service page faults on a data set that
 * lives in pinned host memory and is larger than the frame pool in HBM
 * (paper: System Overview; Paged Memory System Design).  The paper's RDMA-NIC
 * data mover is replaced by the faulting wavefront itself, which copies the
 * page with wide coalesced loads/stores over the host link.
 *
 * Conventions for every entry point:
 *   - returns GPUVM_OK (0) or a negative GPUVM_E* code; gpuvm_strerror() names it;
 *   - "host pointer" = ordinary CPU-addressable memory, "device pointer" = HBM
 *     (e.g. a torch.Tensor's data_ptr()); neither is ever a torch type;
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream);
 *     kernels are enqueued on it; calls that return results to the host
 *     synchronise that stream before returning and say so;
 *   - a gpuvm_t belongs to the device that was current at gpuvm_create() and
 *     may be used by one host thread / one stream at a time.
 */
#ifndef GPUVM_H
#define GPUVM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GPUVM_API __attribute__((visibility("default")))

/* ---- error codes ------------------------------------------------------- */
enum {
    GPUVM_OK      = 0,
    GPUVM_EINVAL  = -1,  /* bad argument (null, size, alignment, policy)        */
    GPUVM_ENOMEM  = -2,  /* device or host allocation failed                    */
    GPUVM_EPIN    = -3,  /* host_buf is not pinned, GPU-mapped host memory      */
    GPUVM_EDEADLK = -4,  /* frame pool too small for the waves a launch needs,
                            or a bounded wait inside a kernel ran out           */
    GPUVM_EHIP    = -5,  /* a HIP runtime call failed                           */
    GPUVM_ERANGE  = -6   /* an index / id array refers outside the data set     */
};

/* ---- eviction policy (paper: Eviction scheme; Oversubscription Analysis) */
enum {
    GPUVM_POLICY_FIFO  = 0, /* ring of frames + reference-counter gate (the paper's) */
    GPUVM_POLICY_CLOCK = 1, /* same ring with a second-chance reference bit          */
    GPUVM_POLICY_CLOCK_WRITE_AWARE = 3, /* CLOCK that spares a DIRTY page one more time
                               before evicting it, so that clean (read-mostly) pages
                               go first and written ones are written back less often
                               (paper: Comparisons with UVM, on write-intensive pages;
                               the paper names the idea, this is one concrete form)   */
    GPUVM_POLICY_GCLOCK = 4, /* generalized CLOCK (not in the paper; the classical GCLOCK
                               with a small counter): a use count of 0..2 per page
                               instead of the bit - installed at 0, raised by every
                               later use, lowered by the passing hand, evicted at 0.
                               Pages earn their chances by being used again, so
                               one-time pages leave first, and a scan never makes
                               the hand pass anything                               */
    GPUVM_POLICY_FIFO_WAIT = 2 /* FIFO, but a leader that draws a frame in use waits
                               (bounded) for its reference counter to reach zero, as
                               the paper words it, instead of passing the frame over;
                               free-running launchers only                           */
};

/* ---- counters ----------------------------------------------------------
 * Wave-aggregated, accumulated since create / gpuvm_stats_clear / gpuvm_reset. */
typedef struct gpuvm_stats {
    uint64_t faults;            /* pages migrated host -> frame                         */
    uint64_t evictions;         /* resident pages dropped to make room                  */
    uint64_t writebacks_evict;  /* dirty victims copied frame -> host                   */
    uint64_t writebacks_flush;  /* dirty pages copied by gpuvm_flush                    */
    uint64_t bytes_in;          /* host-link bytes read by page migration               */
    uint64_t bytes_out;         /* host-link bytes written by write-back                */
    uint64_t hits;              /* page groups that found their page resident           */
    uint64_t wave_page_groups;  /* distinct (wavefront, page) groups after dedup        */
    uint64_t lanes_coalesced;   /* lanes that rode on another lane's group              */
    uint64_t loading_waits;     /* groups that waited for another wave's fault/eviction */
    uint64_t alloc_skips;       /* ring positions passed over: pinned / busy frame      */
    uint64_t alloc_sweeps;      /* CLOCK reference bits cleared by the hand             */
    uint64_t phases;            /* barrier phases run by the deterministic launchers    */
    uint64_t faults_no_fetch;   /* of `faults`: pages installed for a full overwrite,
                                   nothing read from the host                           */
    uint64_t remote_reads;      /* page groups served in place over the link instead of
                                   migrating (gpuvm_set_remote_first)                   */
    uint64_t reserved[1];
} gpuvm_stats_t;

/* ---- device-side view: a POD copied by value into kernel arguments -----
 * (paper: the gpuvm<T> array-like object handed to kernels).  Layout of the
 * tables is described in gpuvm_device.h. */
typedef struct gpuvm_dev {
    unsigned long long *pte;      /* [n_pages] page-table words (device)             */
    unsigned int       *frame_owner; /* [n_frames] page living in the frame          */
    unsigned long long *hand;     /* [0] ring cursor, [1] first error code           */
    unsigned long long *stats;    /* [GPUVM_STAT_SLOTS][16] sharded counters         */
    char               *frames;   /* frame pool, n_frames * page_bytes (device)      */
    char               *host;     /* device-visible address of host_buf              */
    uint64_t bytes;               /* size of the data set                            */
    uint32_t n_pages, n_frames;
    uint32_t page_shift;          /* log2(page_bytes)                                */
    uint32_t policy;
    uint32_t spin_limit;          /* bound on every in-kernel wait loop              */
    uint32_t flags;               /* GPUVM_F_*                                       */
} gpuvm_dev_t;

#define GPUVM_F_ACCESS_STATS 1u   /* also count hits / groups / coalesced lanes     */
#define GPUVM_F_OVERLAPPED_WRITEBACK 2u /* see gpuvm_set_writeback_mode              */
#define GPUVM_F_HANDS_SHIFT 2          /* bits 2..4: two-handed CLOCK, front hand n_frames * value / 8
                                          ahead of the cursor; 0 = one hand (gpuvm_set_clock_hands)  */
#define GPUVM_F_HANDS_MASK 7u
#define GPUVM_F_REMOTE_SHIFT 8         /* flags >> 8: touches in place before a page
                                          migrates, 0 = every miss migrates (see
                                          gpuvm_set_remote_first)                    */
#define GPUVM_STAT_SLOTS 64

typedef struct gpuvm gpuvm_t;     /* opaque; owned by the library */

/* ---- life cycle --------------------------------------------------------- */

/* Pinned, GPU-mapped host memory for a backing store (hipHostMalloc).  The
 * caller owns it and releases it with gpuvm_host_free after gpuvm_destroy. */
GPUVM_API int gpuvm_host_alloc(size_t bytes, void **out);
GPUVM_API int gpuvm_host_free(void *p);

/* Create a paged view of host_buf (paper: Constructing Virtual Memory - the
 * host region is allocated and registered once, before any kernel runs, and
 * its descriptor is copied to the GPU; the GPU pool is allocated statically).
 *   host_buf          host pointer to pinned, GPU-mapped memory (gpuvm_host_alloc,
 *                     hipHostMalloc, or a torch tensor with pin_memory=True);
 *                     stays the caller's, must outlive the handle, and must not
 *                     be touched by the CPU between the first launch and
 *                     gpuvm_flush().  Plain malloc memory -> GPUVM_EPIN.
 *   bytes             size of the data set; the last page may be short.
 *   page_bytes        power of two, 4 KiB .. 1 MiB; every element a launcher
 *                     accesses must not straddle a page.
 *   frame_pool_bytes  HBM budget; n_frames = floor(frame_pool_bytes/page_bytes) >= 2.
 *   policy            GPUVM_POLICY_FIFO, _CLOCK, _CLOCK_WRITE_AWARE, _GCLOCK or _FIFO_WAIT.
 * Allocates (hipMalloc) the frame pool, page table (8 B per page), frame table
 * (4 B per frame) and counters; all pages start INVALID, all frames empty, the
 * ring cursor at 0. */
GPUVM_API int gpuvm_create(void *host_buf, size_t bytes, size_t page_bytes,
                           size_t frame_pool_bytes, int policy, gpuvm_t **out);
GPUVM_API int gpuvm_destroy(gpuvm_t *vm);

/* The same view with its frame pool, page table, frame table, cursor and
 * counters carved out of device memory the caller owns (say, one torch tensor)
 * instead of allocated by the library (paper: Multi-kernel support - the GPU
 * pool is set up once, statically).  gpuvm_workspace_bytes() says how large
 * that memory must be for a given geometry (0 if the geometry is one that
 * gpuvm_create would refuse); d_workspace must be a device pointer on a
 * 256-byte boundary with at least that many bytes (GPUVM_EINVAL otherwise),
 * stays the caller's, must outlive the handle and must not be touched while
 * the handle lives.  gpuvm_destroy() leaves it alone.  Everything else is as
 * for gpuvm_create; the few launchers that keep scratch of their own (the
 * deterministic mode, the edge-balanced graph launchers, the column-order
 * product) still allocate it on first use. */
GPUVM_API size_t gpuvm_workspace_bytes(size_t bytes, size_t page_bytes, size_t frame_pool_bytes);
GPUVM_API int gpuvm_create_in(void *host_buf, size_t bytes, size_t page_bytes, size_t frame_pool_bytes,
                              int policy, void *d_workspace, size_t workspace_bytes, gpuvm_t **out);

/* Copy of the device-side view, for callers that write their own kernels with
 * gpuvm_device.h. */
GPUVM_API int gpuvm_device_handle(const gpuvm_t *vm, gpuvm_dev_t *out);

/* Tuning / test knobs: spin_limit bounds every in-kernel wait (a wave that
 * exceeds it records GPUVM_EDEADLK and the launch returns it; 0 keeps the
 * default); access_stats != 0 turns the per-access counters on. */
GPUVM_API int gpuvm_configure(gpuvm_t *vm, uint32_t spin_limit, int access_stats);

/* How a fault treats a dirty victim.  GPUVM_WB_SERIAL: the paper's
 * order, the write-back completes before the fetch starts.
 * GPUVM_WB_OVERLAPPED: one pass over the frame moves the old content to the
 * host and the new page in, the transfers of both directions in flight
 * together - the obvious remedy for the cost of synchronous write-back that the
 * paper's vector-addition result shows (Evaluation, "Transfer-bound
 * Applications").  Results are the same; only the time of one fault differs,
 * and with a whole wavefront as the mover and other wavefronts filling the
 * link in the meantime the gain is confined to launches with few wavefronts
 * in flight.  Left alone, the library's own launchers that dirty pages use the
 * overlapped order when they keep few wavefronts in flight (at most 64, or
 * at most 256 on pages of 64 KiB and more: the counts up to which the link is
 * not yet full) and the paper's order otherwise; a mode set here is used as it
 * is. */
enum { GPUVM_WB_SERIAL = 0, GPUVM_WB_OVERLAPPED = 1 };
GPUVM_API int gpuvm_set_writeback_mode(gpuvm_t *vm, int mode);

/* One or two hands for the CLOCK policies (GPUVM_POLICY_CLOCK and
 * _CLOCK_WRITE_AWARE; GPUVM_EINVAL for the others unless spread_eighths is 0).
 * With one hand (spread_eighths = 0, the textbook second chance) the cursor
 * clears a set reference bit and passes; since a page is installed with its bit
 * set, a scan - or any pool whose pages are all in use - makes the cursor go
 * round once clearing bits before it finds a victim, every position through
 * the one cursor word.  With two hands (the classical two-handed clock; not in
 * the paper) a front hand n_frames * spread_eighths / 8 positions (1..7 eighths
 * of the ring) ahead of the cursor clears the bit of the frame it stands on every time the cursor
 * advances; the cursor passes a frame only if its page was used again after
 * the front hand went by.  A new page is safe until the cursor has gone once
 * round, a page that is not used again leaves at the cursor's first visit,
 * and a scan makes the cursor pass nothing.  The larger the spread, the longer the time
 * in which a use still counts and the shorter a new page's protection.
 * Default: two hands half a ring apart (spread_eighths = 4).  Takes effect
 * with the next launch. */
#define GPUVM_CLOCK_HANDS_DEFAULT 4
GPUVM_API int gpuvm_set_clock_hands(gpuvm_t *vm, int spread_eighths);

/* Remote-first reads (off by default; not in the paper, whose every miss
 * migrates the page).  A wavefront of this GPU can read pinned host memory in
 * place, so a miss has two prices: the bytes of the access itself over the
 * link, or a whole page.  With bytes_per_touch > 0 a read that misses is
 * served in place and counted in the page's table word; the page migrates
 * once those reads have cost as much as the migration would have
 * (page_bytes / max(bytes_per_touch, 128) touches - the rent-or-buy rule, at
 * most twice the link traffic of knowing the future).  The count starts again
 * when the page is evicted.  bytes_per_touch = what one wavefront reads from a
 * page per access (a 512-byte embedding row, 4 bytes of a gather); 0 turns it
 * off.  Honoured by the element read accessors (gather, filter, products) and
 * the embedding launcher; the edge-balanced graph launchers (BFS, CC, SSSP; set
 * it on the handle of col_idx) use the same trade page by page without a count - a page whose
 * active edge lists would cost less read in place than the page itself is read
 * in place, whatever bytes_per_touch > 0 was given; writes and other page-level
 * users always migrate; the deterministic launchers ignore it.  Results do not change, only traffic:
 * host memory is current for every page that is not resident. */
GPUVM_API int gpuvm_set_remote_first(gpuvm_t *vm, size_t bytes_per_touch);

/* Wavefronts per compute unit the launchers aim for (1..32, default 8; a
 * launch never uses more wavefronts than half the frames).  Left alone, the
 * scatter-increment launcher, whose faults write back as much as they fetch,
 * uses fewer: about 4 MiB of page traffic in flight, where the link's two
 * directions together peak; so do the streaming, embedding and fault-ahead
 * launchers on a pool smaller than the data set (gpuvm_max_waves_streaming).  A value set here (or GPUVM_WAVES_PER_CU in the
 * environment) is used as it is by every launcher. */
GPUVM_API int gpuvm_set_waves_per_cu(gpuvm_t *vm, int waves_per_cu);

/* Synchronise `stream` and return the first error a kernel recorded on this
 * handle since create / reset (GPUVM_OK if none). */
GPUVM_API int gpuvm_check(gpuvm_t *vm, void *stream);

/* Largest number of wavefronts a launcher will keep in flight on this handle:
 * each wave holds at most one pinned page plus one frame under migration, so
 * it is min(n_frames / 2, what the device can hold) - or simply what the device
 * can hold if the pool has a frame for every page, where nothing is ever evicted.  Kernels written against
 * gpuvm_device.h must stay within it too (size the grid from it and stride
 * over the work); beyond it the bounded waits may end a launch with
 * GPUVM_EDEADLK. */
GPUVM_API int gpuvm_max_waves(const gpuvm_t *vm);
/* The same for the launchers whose faults write back as much as they fetch
 * (gpuvm_run_scatter_increment); see gpuvm_set_waves_per_cu. */
GPUVM_API int gpuvm_max_waves_duplex(const gpuvm_t *vm);
/* The same for the launchers that are plain streams of page faults with little
 * work per page (gpuvm_run_stream_reduce, _embedding_bag, _prefetch): on a pool
 * smaller than the data set they keep about 4 MiB of page traffic in flight,
 * which fills the link; more only queues in front of the other memory traffic.
 * On a pool that holds every page - hits only, after the first touch - they
 * run 16 wavefronts per compute unit, where reads of resident pages come
 * closest to a plain read of HBM. */
GPUVM_API int gpuvm_max_waves_streaming(const gpuvm_t *vm);

/* Write every DIRTY page back to host_buf and clear the dirty bits; pages stay
 * resident (not in the paper, whose write-back happens only at eviction:
 * Transfer-bound Applications).  Synchronises `stream`; afterwards host_buf is
 * authoritative and the CPU may read it. */
GPUVM_API int gpuvm_flush(gpuvm_t *vm, void *stream);

/* gpuvm_flush, then forget every mapping: cold start (all INVALID, frames
 * empty, cursor 0) and zeroed counters.  Synchronises `stream`. */
GPUVM_API int gpuvm_reset(gpuvm_t *vm, void *stream);

/* Sum the sharded device counters into *out (host pointer).  Synchronises the
 * device. */
GPUVM_API int gpuvm_stats(gpuvm_t *vm, gpuvm_stats_t *out);
GPUVM_API int gpuvm_stats_clear(gpuvm_t *vm);

/* Copy the raw tables to host arrays for invariant checks: pte_out[n_pages]
 * (see gpuvm_device.h for the bit layout), owner_out[n_frames] (0xFFFFFFFF =
 * empty), *hand_out = ring cursor.  Any pointer may be NULL.  Synchronises. */
GPUVM_API int gpuvm_dump_tables(gpuvm_t *vm, uint64_t *pte_out, uint32_t *owner_out,
                                uint64_t *hand_out);

GPUVM_API const char *gpuvm_strerror(int code);

/* ---- workload launchers (free-running fault handling) --------------------
 * Each runs the whole hot path - address split, page-table lookup with
 * reference count, wavefront dedup, inter-wave fault arbitration, frame
 * allocation with eviction and dirty write-back, page migration, access,
 * unpin (paper: System Overview steps 1-7; Paged Memory System Design) -
 * inside its kernel.  All array arguments are device pointers.  Launches are
 * asynchronous on `stream` unless stated; a kernel-side GPUVM_EDEADLK is
 * reported by the next synchronising call on the handle.
 * Launches on one handle must be ordered one after the other (same stream, or
 * events): each is sized so that its wavefronts can hold at most half of the
 * frames at once, which is what guarantees progress; two launches running
 * together on one handle may exceed that, and then the bounded waits end them
 * with GPUVM_EDEADLK instead of hanging.  Different handles are independent. */

/* Random gather over a uint32 data set: out[k] = data[idx[k]], *sum += sum_k out[k]
 * (d_sum: one uint64 in device memory, accumulated with atomics; may be NULL).
 * idx values must be < bytes/4 (checked in the kernel: GPUVM_ERANGE). */
GPUVM_API int gpuvm_run_gather(gpuvm_t *vm, const uint32_t *d_idx, size_t n,
                               uint32_t *d_out, uint64_t *d_sum, void *stream);

/* The gather above and the scatter-increment below for thread-per-element code
 * with a condition around the access (the style of the paper's listing): element k takes part only if
 * d_mask[k] != 0 (one byte per element, device memory), and only those lanes
 * enter the accessors, so the fault path runs under arbitrary divergence.
 *   gather:    out[k] = data[idx[k]] for the masked k; other out[k] untouched.
 *   increment: data[idx[k]] += 1 (uint64 elements) for the masked k.
 * Index bounds as for the unmasked forms (GPUVM_ERANGE from the kernel). */
GPUVM_API int gpuvm_run_gather_masked(gpuvm_t *vm, const uint32_t *d_idx, const uint8_t *d_mask,
                                      size_t n, uint32_t *d_out, void *stream);
GPUVM_API int gpuvm_run_scatter_increment_masked(gpuvm_t *vm, const uint32_t *d_idx,
                                                 const uint8_t *d_mask, size_t n, void *stream);

/* The paper's vector-addition listing: C[i] = A[i] + B[i] for i < n over three
 * paged fp32 vectors (three handles, each with its own frame pool; A and B may
 * be the same handle, C must be distinct).  C is written with gpuvm_store, its
 * pages become DIRTY and reach the host at eviction or gpuvm_flush(vm_c). */
GPUVM_API int gpuvm_run_vector_add(gpuvm_t *vm_a, gpuvm_t *vm_b, gpuvm_t *vm_c, size_t n,
                                   void *stream);

/* The same result with C's pages taken through gpuvm_acquire_overwrite: a
 * wavefront owns one page of C at a time and stores all of it, so a miss on C
 * installs a frame without reading the page from the host first - 8 of the 12
 * bytes per element cross the link inwards instead of 12.  Not in the paper
 * (its write faults fetch).  Same arguments and errors as above; in addition
 * C[0..n) must end on a page boundary of C or where C ends (GPUVM_EINVAL
 * otherwise: a page stored only in part would need its old content). */
GPUVM_API int gpuvm_run_vector_add_overwrite(gpuvm_t *vm_a, gpuvm_t *vm_b, gpuvm_t *vm_c, size_t n,
                                   void *stream);

/* Fault-ahead of pages [first_page, first_page + n_pages): every page of the
 * range that is not resident is migrated (evicting as usual), nothing is read
 * from it.  The counterpart of the prefetch hints the paper applies to its UVM
 * baseline (Evaluation), for callers that know what the next kernel will
 * touch; a range larger than the pool only turns the pool over.
 * GPUVM_ERANGE if the range leaves the data set. */
GPUVM_API int gpuvm_run_prefetch(gpuvm_t *vm, size_t first_page, size_t n_pages, void *stream);

/* One pass of a streaming read-reduce over an fp32 data set: for each block of
 * block_elems consecutive floats (a multiple of the page's float count),
 * d_sums[b] = sum in fp64.  One wavefront per page, consecutive pages to
 * consecutive wavefronts. */
GPUVM_API int gpuvm_run_stream_reduce(gpuvm_t *vm, size_t block_elems,
                                      double *d_sums, void *stream);

/* Level-synchronous BFS; the data set is the int32 col_idx array of a CSR
 * graph, d_row_ptr[nv+1] (int64) and d_level[nv] (int32 out, -1 = unreachable)
 * are plain device memory.  One kernel per level; synchronises `stream`
 * between levels.  *n_levels_out (host, may be NULL) = number of levels run. */
GPUVM_API int gpuvm_run_bfs(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv,
                            int64_t src, int32_t *d_level, int *n_levels_out,
                            void *stream);

/* The same BFS with the work cut into equal chunks of edges instead of
 * vertices (paper: Graph Workloads, Balanced CSR - an even number of faults
 * per worker, no serialisation behind huge neighbour lists): a wavefront owns
 * one page of col_idx per level and walks the segments of the frontier's
 * vertices inside it.  A level visits only the pages that hold edges of its
 * frontier, and starts with those of them that the level before left in the
 * pool (paper: Multi-kernel support - mappings persist from kernel to
 * kernel): the resident pages are taken in the order in which the allocator
 * would evict them, two for every page that has to be faulted in.  Same
 * arguments and result as gpuvm_run_bfs; the row_ptr array must be
 * non-decreasing with row_ptr[nv] = bytes / 4.  The CC and SSSP launchers
 * below walk their rounds the same way. */
GPUVM_API int gpuvm_run_bfs_balanced(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv,
                                     int64_t src, int32_t *d_level, int *n_levels_out,
                                     void *stream);

/* Weakly connected components on the same paged CSR graph, edge-balanced like
 * gpuvm_run_bfs_balanced (paper: Graph Workloads evaluates BFS, CC and SSSP):
 * label propagation until nothing changes; every round reads every edge.
 * d_label[nv] (int32 out) = smallest vertex id of the vertex's component.
 * *n_rounds_out (host, may be NULL) = rounds run.  Synchronises per round. */
GPUVM_API int gpuvm_run_cc_balanced(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv,
                                    int32_t *d_label, int *n_rounds_out, void *stream);

/* Single-source shortest paths with uint32 edge weights that are paged from
 * host memory as a second data set (paper: SSSP pages edges + weights):
 * vm_weights is a handle over a uint32 array parallel to col_idx (same byte
 * size and page size as vm, its own frame pool).  A wave holds one page of
 * each handle at a time.  d_dist[nv] (uint32 out) = distance from src,
 * 0xFFFFFFFF if unreachable; path lengths must stay below 2^32 - 1.
 * Frontier-based Bellman-Ford rounds; synchronises per round. */
GPUVM_API int gpuvm_run_sssp_balanced(gpuvm_t *vm, gpuvm_t *vm_weights, const int64_t *d_row_ptr,
                                      int64_t nv, int64_t src, uint32_t *d_dist,
                                      int *n_rounds_out, void *stream);

/* Embedding-bag lookup with sum pooling over an fp32 table of `dim` columns
 * (dim * 4 bytes must divide page_bytes; dim a multiple of 64 up to 256):
 * d_out[bag][c] = sum_j table[d_ids[bag][j]][c], rows added in listed order in
 * fp32.  ids must be in [0, bytes/(4*dim)). */
GPUVM_API int gpuvm_run_embedding_bag(gpuvm_t *vm, size_t dim, const int32_t *d_ids,
                                      size_t bags, size_t bag_len, float *d_out,
                                      void *stream);

/* y = A^T x over a paged row-major fp32 matrix A[rows][cols] (rows * cols * 4
 * = bytes): one thread per column walking down the rows - the column-order
 * access of the paper's transfer-bound applications (MVT / ATAX pattern).
 * d_x[rows] fp32, d_y[cols] fp64 out (fp64 accumulation, rows ascending). */
GPUVM_API int gpuvm_run_matvec_t(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x,
                                 double *d_y, void *stream);

/* gpuvm_run_matvec_t for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, result and errors; it calls no hipMalloc / hipFree and no other
 * allocating routine.  The one scratch buffer of the product (the row every
 * compute wavefront has reached, 4 bytes per wavefront, which the other entry
 * point allocates per handle on first use) lives in a static device array of
 * GPUVM_NOALLOC_MAX_COLS / 64 words = 8 KiB that every GPU the library runs on
 * holds until the process ends.  cols above GPUVM_NOALLOC_MAX_COLS are refused
 * with GPUVM_ERANGE (and a line on stderr).  The handle's device must be the
 * current one (GPUVM_EINVAL otherwise).  All calls on one GPU share the array:
 * it is cleared by a fill kernel at the start of every call, and calls that
 * overlap on one GPU (different streams, different handles) race on it - order
 * them.  The caller still passes inputs and outputs; the handle was created
 * (and its pool allocated) beforehand. */
#define GPUVM_NOALLOC_MAX_COLS 131072
GPUVM_API int gpuvm_run_matvec_t_noalloc(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x,
                                         double *d_y, void *stream);

/* y = A x over the same kind of matrix, one thread per ROW (the first product
 * of the paper's MVT, the first step of its ATAX): the lanes of a wavefront
 * stand on 64 different pages and walk along their rows.  cols must be a
 * multiple of 4 and rows * cols * 4 = bytes (GPUVM_EINVAL otherwise); d_x[cols]
 * fp32, d_y[rows] fp64 out (fp64 accumulation, columns ascending).  The
 * launcher keeps the rows in flight within 3/4 of the pool. */
GPUVM_API int gpuvm_run_matvec(gpuvm_t *vm, size_t rows, size_t cols, const float *d_x,
                               double *d_y, void *stream);

/* Filter-then-gather over two paged uint32 columns of equal length (paper:
 * Query Evaluation Benchmarks - scan one column, fetch another only for the
 * rows that pass): *d_count = #{i : key[i] > threshold}, *d_sum = sum of
 * val[i] over those rows (both one uint64 in device memory, overwritten). */
GPUVM_API int gpuvm_run_filter_sum(gpuvm_t *vm_key, gpuvm_t *vm_val, uint32_t threshold,
                                   uint64_t *d_count, uint64_t *d_sum, void *stream);

/* Scatter-increment over a uint64 data set: data[idx[k]] += 1 (device atomics
 * on the frame; pages become DIRTY and reach host_buf at eviction or flush). */
GPUVM_API int gpuvm_run_scatter_increment(gpuvm_t *vm, const uint32_t *d_idx,
                                          size_t n, void *stream);

/* ---- deterministic barrier-phased launchers ------------------------------
 * The same work cut into phases of phase_len consecutive accesses; inside a
 * phase: (A) all waves dedup, pin resident pages and list missing ones,
 * (B) one sequential agent serves the missing pages in ascending page order,
 * walking the ring exactly like a sequential replay, (C) all waves migrate the
 * assigned pages in parallel, (D) access and unpin.  Fault / eviction /
 * write-back counts and the final frame table are then unique and must equal
 * a sequential FIFO / CLOCK replay.  A phase may touch at most n_frames
 * distinct pages (else GPUVM_EDEADLK).  Synchronise `stream` before returning. */
GPUVM_API int gpuvm_run_gather_phased(gpuvm_t *vm, const uint32_t *d_idx, size_t n,
                                      size_t phase_len, uint32_t *d_out,
                                      uint64_t *d_sum, void *stream);
GPUVM_API int gpuvm_run_scatter_increment_phased(gpuvm_t *vm, const uint32_t *d_idx,
                                                 size_t n, size_t phase_len,
                                                 void *stream);

/* ---- roofline microbenchmarks ---------------------------------------------
 * The paper's transfer benchmark (Comparison with GPUDirect RDMA: a large
 * buffer streamed with one page per warp) recast for the wavefront mover:
 * copy `bytes` from src to dst in chunks of chunk_bytes, one chunk per
 * wavefront at a time, with `waves` wavefronts in total (0 = as many as the
 * device holds).  src/dst are device-visible pointers (HBM, or pinned host
 * memory for the host-link directions).  Asynchronous on `stream`. */
GPUVM_API int gpuvm_bench_copy(void *dst, const void *src, size_t bytes,
                               size_t chunk_bytes, int waves, void *stream);

/* The same copy with the data staged through LDS instead of registers (eight
 * direct-to-LDS loads of 1 KiB per wavefront in flight, then LDS reads and
 * stores): the other way to build the page mover, kept so that the two can be
 * measured side by side (paper: Register usage - the runtime is inlined into
 * every kernel, so what the mover holds in registers is every kernel's cost).
 * bytes and chunk_bytes are multiples of 16; otherwise as gpuvm_bench_copy. */
GPUVM_API int gpuvm_bench_copy_lds(void *dst, const void *src, size_t bytes,
                                   size_t chunk_bytes, int waves, void *stream);

/* Same traffic, reading only (every lane folds what it loaded into one word of
 * d_sink so the loads cannot be dropped): the read-side link / HBM ceiling. */
GPUVM_API int gpuvm_bench_read(const void *src, size_t bytes, size_t chunk_bytes,
                               int waves, uint64_t *d_sink, void *stream);

/* Unloaded round-trip time of one 1 KiB wavefront load from src (device-visible
 * pointer, 1 MiB <= bytes <= 2 GiB): one wave, `hops` dependent loads.
 * *ns_per_hop_out is a host pointer.  Synchronises `stream`.  With the
 * bandwidth above it gives the bytes that must be in flight to fill the link
 * (paper: Efficient RDMA I/O Management, the queue-depth argument). */
GPUVM_API int gpuvm_bench_latency(const void *src, size_t bytes, int hops, double *ns_per_hop_out,
                                  void *stream);

/* Zero-copy baseline of gpuvm_run_bfs_balanced: the same edge-balanced kernel
 * reading col_idx in place in the handle's pinned host buffer, with no page
 * table and no frames (direct access, the alternative to demand paging on a
 * GPU whose wavefronts can address host memory).  Same arguments and result;
 * the handle only names the buffer
 * and its page geometry, its tables and counters are not touched. */
GPUVM_API int gpuvm_bench_bfs_zero_copy(gpuvm_t *vm, const int64_t *d_row_ptr, int64_t nv, int64_t src,
                                        int32_t *d_level, int *n_levels_out, void *stream);

/* The same for gpuvm_run_embedding_bag: rows are read in place in the pinned
 * host buffer, 64 lanes on one contiguous row. */
GPUVM_API int gpuvm_bench_embedding_bag_zero_copy(gpuvm_t *vm, size_t dim, const int32_t *d_ids,
                                                  size_t bags, size_t bag_len, float *d_out,
                                                  void *stream);

/* Plain device-resident random gather with no page table (the ceiling for
 * hits): out[k] = data[idx[k]]. */
GPUVM_API int gpuvm_bench_gather_plain(const uint32_t *d_data, const uint32_t *d_idx,
                                       size_t n, uint32_t *d_out, void *stream);

/* Plain scatter-increment with no page table: data[idx[k]] += 1 on a uint64
 * array, with system-scope atomics.  `data` in device memory: the ceiling for
 * hits of the scatter workload; `data` in pinned host memory: its zero-copy
 * form, every update an atomic executed over the link.  idx values must be
 * below the array's length (not checked). */
GPUVM_API int gpuvm_bench_scatter_plain(uint64_t *data, const uint32_t *d_idx, size_t n, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GPUVM_H */
