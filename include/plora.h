/* plora.h - C ABI of the paged multi-LoRA library for MI355X (gfx950).
 *
 * The library computes the heterogeneous-rank multi-LoRA delta of Predictive-LoRA: for every
 * token t of a batch whose adapter is i,
 *        y[t,:] += scale_i * (x[t,:] * A_i^T) * B_i
 * (Sec. II-A, Eq. 1: W = W0 + B A; stored orientation below), where A_i and B_i live in a pool
 * of fixed-size GPU pages and are gathered through a per-adapter page table (Sec. III-C "Page
 * Structure", "Page Table"; Sec. IV "Memory Manager").  Around the two kernels sit the page
 * allocator that places and evicts adapters (Sec. III-C; Sec. III-B "Eviction Policy",
 * mechanism only) and the pinned-host -> GPU copy that fills the pages (Sec. III-B "Prefetch
 * Scheduling").
 *
 * Conventions
 *  - Every call returns a plora_status; a failed call leaves the pool unchanged.
 *  - "host" / "device" is stated for every pointer.  Streams are hipStream_t values passed as
 *    plain pointers (plora_stream); NULL is the null stream.
 *  - A *slot* is one linear map d_in -> d_out that every adapter of the pool covers.  An adapter of
 *    rank r is one contiguous blob of  S = r * elt * sum_slots(d_in + d_out)  bytes, slot after
 *    slot, each slot as [A_s | B_s] with A_s = r rows of d_in elements and B_s = r rows of d_out
 *    elements (both rank-major, no padding).  A_s is the paper's A; B_s is the paper's B transposed.
 *  - The blob occupies ceil(S / page_bytes) pages: the lowest-numbered free pages, in ascending
 *    order (first fit).  Virtual byte o of the blob lives at slab + pt[o / P] * P + o % P.
 *  - Not thread safe: one host thread drives a pool.
 */
#ifndef PLORA_H
#define PLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct plora_pool plora_pool;   /* opaque, owned by the library */
typedef struct plora_batch plora_batch; /* opaque, owned by the pool that made it */
typedef void* plora_stream;             /* a hipStream_t */

typedef enum {
  PLORA_OK = 0,
  PLORA_ERR_INVAL = -1,    /* bad argument, alignment, rank, id or size */
  PLORA_ERR_NOMEM = -2,    /* fewer free pages than needed; nothing was allocated */
  PLORA_ERR_EXISTS = -3,   /* id already resident (or still loading) */
  PLORA_ERR_NOTFOUND = -4, /* id not resident */
  PLORA_ERR_BUSY = -5,     /* evict of an adapter whose load has not completed or that an open batch uses */
  PLORA_ERR_HIP = -6,      /* a HIP runtime call failed; see plora_last_hip */
  PLORA_ERR_LIMIT = -7     /* the request is valid but larger than a fixed capacity of the entry point */
} plora_status;

typedef enum { PLORA_F16 = 0, PLORA_BF16 = 1, PLORA_F32 = 2 } plora_dtype;

typedef struct {
  int32_t n_slots;      /* 1 .. 32767 */
  const int32_t* d_in;  /* host, n_slots entries, each > 0 and a multiple of 8 */
  const int32_t* d_out; /* host, n_slots entries, each > 0 and a multiple of 8 */
  int32_t dtype;        /* plora_dtype of weights, x and y */
  int32_t max_adapters; /* adapter ids are 0 .. max_adapters-1 */
  int32_t max_rank;     /* 1 <= rank <= max_rank <= 512; also the row stride of v */
} plora_layout;

/* plora_pool_create flags */
#define PLORA_POOL_PLACEMENT_ONLY 1u /* allocator and batch translation only: no device memory, no
                                        copies; shrink / expand return PLORA_ERR_INVAL.  For capacity
                                        planning and host-side tests on a machine without a GPU. */

typedef struct {
  uint64_t page_bytes, n_pages, used_pages, free_pages;
  uint64_t resident_adapters;
  uint64_t resident_bytes;      /* sum of S over resident adapters */
  uint64_t internal_frag_bytes; /* used_pages * page_bytes - resident_bytes */
  uint64_t loads, evictions, nomem_failures;
  uint64_t h2d_bytes;  /* bytes handed to the copy engine by plora_load_adapter */
  uint64_t h2d_copies; /* number of copy calls (one per run of physically consecutive pages) */
  double h2d_ms;       /* summed first-copy-start -> last-copy-end time of completed loads */
  uint64_t staged_loads; /* loads that went through a staging buffer and the scatter kernel */
  uint64_t fused_launches; /* plora_delta calls that ran as one launch */
  uint64_t fused_timeouts; /* expand tasks of such launches that gave up waiting for their slot's shrink tasks (their
                              part of y was left as it was); stays 0 unless "fused_spin_limit" is set very low */
  uint64_t compacted_adapters, compacted_pages; /* moved by plora_compact so far */
  double compact_ms;       /* summed first-copy-start -> last-copy-end time of completed moves */
} plora_stats;

/* Pool of n_pages pages of page_bytes each (Sec. III-C "Page Structure"; the paper's default page is
 * 2 MB).  page_bytes: power of two >= 4096.  slab_or_null: device pointer to at least
 * n_pages * page_bytes bytes, 256-byte aligned, that stays valid until plora_pool_destroy (the
 * caller keeps ownership), or NULL to let the pool allocate and own the slab.  The layout arrays are
 * copied.  INVAL for bad sizes or a layout whose rows would need more page-table window than the
 * kernels stage (32 * max(d_in) * elt / page_bytes + 8 > 1024). */
int plora_pool_create(size_t page_bytes, uint32_t n_pages, const plora_layout* layout, void* slab_or_null,
                      uint32_t flags, plora_pool** out);

/* Frees everything the pool owns.  Synchronises the device first.  BUSY if a batch is still open. */
int plora_pool_destroy(plora_pool* pool);

/* Bytes of a rank-`rank` adapter blob for this pool's layout (0 if rank is out of range). */
uint64_t plora_adapter_bytes(const plora_pool* pool, int32_t rank);

/* Place adapter `id` and start filling its pages (Sec. III-B: load from host memory to GPU;
 * Sec. III-C: ceil(S/P) pages).  pinned_host_ptr: host, page-locked, S bytes, must stay valid and
 * unchanged until the adapter is ready.  The copies are issued on copy_stream, one per run of
 * physically consecutive pages (or, with the option "staging_bytes", one copy into a staging buffer
 * and a kernel that moves the pages into place), after that stream has been made to wait for every batch, on whatever
 * stream it ran, that read since-freed pages and has not finished (copy streams may differ from
 * load to load).  page_table_out / n_pages_out (either may be NULL): the adapter's
 * page table, a host pointer into pool-owned memory that stays valid until plora_evict(id).
 * Returns at once; the adapter becomes usable by batches immediately (they wait on its ready event).
 * INVAL (bad id / rank / pointer not page-locked), EXISTS, NOMEM (nothing allocated). */
int plora_load_adapter(plora_pool* pool, int32_t id, int32_t rank, float scale, const void* pinned_host_ptr,
                       plora_stream copy_stream, const int32_t** page_table_out, uint32_t* n_pages_out);

/* 1 if the adapter's copies have completed, 0 if still in flight, or a negative plora_status. */
int plora_adapter_ready(plora_pool* pool, int32_t id);

/* Makes `stream` wait (device side) until the adapter's copies have completed. */
int plora_wait_adapter(plora_pool* pool, int32_t id, plora_stream stream);

/* Blocks the calling host thread until the adapter's copies have completed. */
int plora_sync_adapter(plora_pool* pool, int32_t id);

/* Return the adapter's pages to the free set (Sec. III-B "Eviction Policy": the mechanism).  The
 * pages are allocatable at once.  NOTFOUND; BUSY if the load has not completed or an open batch
 * names the adapter. */
int plora_evict(plora_pool* pool, int32_t id);

/* The adapter's current page table (Sec. III-C "Page Table"): the same pool-owned array that
 * plora_load_adapter handed out, n_pages entries, valid until plora_evict(id); plora_compact rewrites it
 * in place.  NOTFOUND. */
int plora_adapter_pages(plora_pool* pool, int32_t id, const int32_t** page_table_out, uint32_t* n_pages_out);

/* Compaction (Sec. III-C "Defragmentation": background compaction coalesces free pages).  With pages of
 * one size no allocation can fail for lack of a contiguous range; what scattered free pages cost is one
 * copy per run of consecutive pages when an adapter is loaded, and a table read at the head of every
 * work item of an adapter that is not on consecutive pages.  The call takes the resident adapters in
 * ascending order of their first page and places each anew where a load would put it if its own pages
 * were free as well - on the lowest-numbered pages among the free ones and its own, ascending -
 * moving its pages there with device-to-device copies on `stream`.  Adapters that an open batch names
 * or whose load has not completed stay where they are.  max_pages > 0 bounds the pages moved by one
 * call (a background step): an adapter moves whole or not at all, and the first that does not fit ends
 * the call.  pages_moved_out / adapters_moved_out (host, may be NULL).
 * Ordering: the copies wait (device side) for every batch still in flight that reads pages they write,
 * on whatever stream it ran; batches begun afterwards wait for the moved adapter like for a load in
 * flight (plora_adapter_ready / plora_wait_adapter apply); whoever writes the vacated pages next waits
 * for the copies and for the batches that still read them.  Results of batches do not change.
 * PLORA_ERR_HIP: the adapter whose move failed has left the pool (its pages may have been overwritten
 * half way) and has to be loaded again; adapters moved before it stay moved. */
int plora_compact(plora_pool* pool, plora_stream stream, uint32_t max_pages, uint32_t* pages_moved_out,
                  uint32_t* adapters_moved_out);

/* Once-per-batch translation (Sec. III-C "Page Table").  tok2adapter_host: host, n_tokens entries;
 * -1 = token without adapter (its y row is left untouched).  Groups tokens by adapter with a stable
 * counting sort (ascending adapter id), resolves each group's rank, scale and page table, builds the
 * work lists of the kernels and sends all of it to the device with one copy on `stream`; `stream`
 * is also made to wait for the adapters' copies.  The adapters named are pinned against eviction
 * until plora_batch_end.  n_tokens may be 0.  NOTFOUND if a token names a non-resident adapter,
 * INVAL for ids outside [-1, max_adapters). */
int plora_batch_begin(plora_pool* pool, const int32_t* tok2adapter_host, int32_t n_tokens, plora_stream stream,
                      plora_batch** out);

/* The translation's result, for inspection: perm (token indices sorted by adapter, n_perm entries),
 * seg_adapter (n_seg distinct ids, ascending), seg_start (n_seg + 1 offsets into perm).  Host
 * pointers owned by the batch, valid until plora_batch_end.  Any out pointer may be NULL. */
int plora_batch_info(const plora_batch* batch, int32_t* n_seg, int32_t* n_perm, const int32_t** perm,
                     const int32_t** seg_adapter, const int32_t** seg_start);

/* Shrink, slots slot0 .. slot0+n_slots-1, one launch sequence for all of them:
 *   v[s][t, j] = sum_k x[s][t,k] * A_i[j,k]   (j < r_i, i = adapter of t; fp32 accumulation)
 *   v[s][t, j] = 0                            (r_i <= j < max_rank, or t has no adapter)
 * x: host array of n_slots device pointers, x[q] -> n_tokens x d_in[slot0+q] elements, row-major,
 * 16-byte aligned.  v: host array of n_slots device pointers, v[q] -> n_tokens x max_rank floats,
 * 16-byte aligned.  Runs on `stream`: normally the stream given to plora_batch_begin; another stream
 * must be ordered after that one by the caller (the batch's tables arrive on it), and plora_batch_end
 * then makes the batch's own stream wait for the other stream's kernels, so that later evictions and
 * loads are ordered after every kernel of the batch.  While plora_profile is off, plora_shrink and
 * plora_expand call no device allocator and enqueue kernels only, so they may be recorded into a HIP
 * graph on a capturing stream; the batch has to stay open, and x, v, y in place, for as long as the
 * graph is replayed, and plora_batch_end must not be called while such a stream is still capturing. */
int plora_shrink(plora_pool* pool, const plora_batch* batch, int32_t slot0, int32_t n_slots, const void* const* x,
                 float* const* v, plora_stream stream);

/* Expand, same slot range:
 *   y[s][t, n] = round_to_elt( y[s][t,n] + scale_i * sum_j v[s][t,j] * B_i[j,n] )   (fp32 accumulation,
 * one rounding to nearest even).  y: host array of n_slots device pointers, y[q] -> n_tokens x
 * d_out[slot0+q] elements, row-major, 16-byte aligned, updated in place. */
int plora_expand(plora_pool* pool, const plora_batch* batch, int32_t slot0, int32_t n_slots, const float* const* v,
                 void* const* y, plora_stream stream);

/* Eq. 1's delta in one call: shrink, then expand, over the same slot range, as plora_shrink followed by
 * plora_expand with the same arguments would do (v is the workspace in between; its contents afterwards
 * are those plora_shrink leaves).  Nothing is queued if an argument is invalid.  With the option
 * "fused_max_tasks" set, a call on the batch's own stream of at most 32 slots and that many workgroups'
 * worth of work (not a batch of large groups, not a stream under graph capture) runs as ONE launch: the
 * workgroups of a persistent grid run the shrink and then the expand work, an expand task waiting
 * (bounded) until its slot's shrink tasks have finished; results are bit-identical to the two-launch
 * form.  Such launches on one batch must not overlap, which the single stream guarantees. */
int plora_delta(plora_pool* pool, const plora_batch* batch, int32_t slot0, int32_t n_slots, const void* const* x,
                float* const* v, void* const* y, plora_stream stream);

/* plora_delta for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): the workspace v lives in a static device array of the
 * library, 16 MiB per GPU, held from the library's first use on that GPU until the process ends.
 * Calls no allocator of the HIP runtime (nor any host allocator).  LIMIT if
 * n_slots * round_up(n_tokens * max_rank * 4, 256) exceeds 16 MiB; INVAL while plora_profile is on.
 * Every call on a GPU uses the same array from its start: two calls whose kernels may overlap on
 * one GPU (different streams, or two pools) race; calls on one stream are ordered and safe.  x and y
 * as in plora_shrink / plora_expand. */
int plora_delta_static(plora_pool* pool, const plora_batch* batch, int32_t slot0, int32_t n_slots,
                       const void* const* x, void* const* y, plora_stream stream);

/* Ends the batch: unpins its adapters, hands the batch object back for reuse and notes that its
 * completion has to be recorded on its stream (the stream given to plora_batch_begin).  Kernels
 * already enqueued keep running; pages freed afterwards are not overwritten before they finish.
 * The record itself may be put on the stream later, by this or a later call into the library (see
 * the option "batches_per_marker"): a stream that batches ran on must therefore stay valid until
 * the pool is destroyed, or the option be set to 1, which records inside this call. */
int plora_batch_end(plora_pool* pool, plora_batch* batch);

/* Counters of the pool (Sec. V-A lists memory utilisation and fragmentation as metrics). */
int plora_pool_stats(plora_pool* pool, plora_stats* out);

/* Tunables.  An adapter group of n tokens and rank r uses the matrix-core items when n >=
 * "mfma_min_tokens" / "mfma_min_tokens_expand" (shrink / expand; defaults 16 / 64; 0 = never, 1 =
 * always) or when its work reaches "mfma_min_work" / "mfma_min_work_expand" (defaults 64 / 128; 1 ..
 * 2^30), where work = n * r for shrink and n * r * r / (r rounded up to a multiple of 32) for expand;
 * they take effect for batches begun afterwards.  "slot_major" (-1 =
 * slots are the fastest grid dimension when their count is a multiple of 8, 0 never, 1 always; for
 * expand also 2 = the 512-column chunks of one work item are the fastest dimension, so that
 * neighbouring workgroups read neighbouring pieces of the same rows of B) and "xcd_remap" (1 = for
 * launches whose fastest dimension is not the slot, neighbouring work items share an XCD) set the
 * launch geometry of both operations; with the suffix "_shrink" / "_expand" of one (defaults: shrink
 * -1 and 1, expand 2 and 0).  "coop_max_workgroups_shrink" / "coop_max_workgroups_expand" (a call
 * whose ordinary launch would have at most this many workgroups is too small to fill the GPU and bound
 * by its longest chain of dependent loads; it runs the cooperative kernels instead, in which the four
 * wavefronts of a workgroup share one vector-ALU item; defaults 192 / 2500, 0 = never; take effect for
 * batches begun afterwards).  "batches_per_marker" (1..64, default 4: plora_batch_end puts one completion
 * event on the stream per this many batches instead of one per batch; the library records a pending
 * one itself whenever an eviction, a load or the reuse of a batch object has to order against it, so
 * the value changes only how long pages and batch objects may stay held, never results).
 * "panel_min_blocks" (>= 0, default 8): expand cuts the large adapter groups of a batch into blocks of
 * 64 tokens and runs them in a kernel that holds a panel of B in LDS when the batch has at least this
 * many such blocks (prefill); other batches (decode: a hot adapter or two) cut them into items of 16
 * tokens for the ordinary kernel instead (0 = always).  "mfma_cols_max_group" (default 32): in a
 * batch of the first kind, a group's last <= this many tokens still go as 16-token items.
 * "panel_half_max_workgroups" (>= 0, default 8192): a launch of that kernel with at most this many
 * workgroups of 512 columns is issued with one workgroup per 256 columns instead (twice as many, each
 * half as long; v is then read twice as often), which is faster while the launch is too short to hide
 * a workgroup's chain of loads behind other workgroups; 0 = never.  Results do not depend on it.
 * "mfma_shrink_depth" (0, 1 or 2; default 0): runs of 64 values of the contraction that a matrix-core
 * shrink item keeps in flight per wavefront; 0 lets the library choose per launch (2 when the batch's
 * matrix-core token tiles are at least half full on average, as in prefill, when a slot of the launch
 * has d_in > 4096, or when the launch has at most 2500 workgroups; else 1).  Results do not depend on it.
 * "contig_fast_path" (0 or 1, default 1; for adapters loaded afterwards): an adapter whose pages are
 * physically consecutive is handed to the kernels by its first page instead of its page table (no table
 * entries in the batch's image, one dependent read less at the head of every work item); 0 treats every
 * adapter alike.  Results do not depend on it.
 * "fused_max_tasks" (0 .. 2^30, default 0 = never): plora_delta calls of at most this many workgroup
 * tasks run as one launch (see plora_delta; measured slower than the two launches on MI355X at every call
 * size, hence off).  "fused_spin_limit" (0 .. 2^31, default 2^20): polls of a
 * slot's completion counter before an expand task of such a launch gives up (counted in
 * plora_stats.fused_timeouts); only a test has reason to lower it.
 * "staging_bytes" (0 .. 2^36, default 0 = off) and "staging_min_runs" (>= 1, default 3: with two runs the direct copies are as fast): staged loads
 * (Sec. III-B: loaded adapters arrive in a staging area before they are moved into place).  With
 * staging on, plora_load_adapter sends a blob of at most staging_bytes whose pages form at least
 * staging_min_runs runs of consecutive pages in ONE copy into one of two device staging buffers of
 * staging_bytes each (allocated by this call, which synchronises the device when it has to grow
 * them) and lets a kernel on copy_stream move the pages into place; that copy does not have to wait
 * for earlier readers of the freed pages, only the kernel does.  Other blobs keep the direct path.
 * INVAL for an unknown key or a value out of range (staging_bytes: also for a placement-only pool). */
int plora_pool_set_option(plora_pool* pool, const char* key, int64_t value);

/* Kernel timing for benchmarks.  plora_profile(pool, 1) makes plora_shrink / plora_expand attach a
 * pair of HIP events to the kernel dispatches of every call (start of its first kernel, end of its
 * last; nothing extra is queued on the stream); plora_profile(pool, 0) stops.
 * plora_profile_read waits for the recorded events and returns, per kernel class (0 shrink, 1 expand,
 * 2 the one-launch form of plora_delta), the summed duration in ms and the number of launches since the
 * last read, then clears the record.  ms and launches: host, 3 entries each. */
int plora_profile(plora_pool* pool, int enable);
int plora_profile_read(plora_pool* pool, double* ms, uint64_t* launches);

/* ---------------------------------------------------------------------------------------------
 * Residency policy (Sec. III-B), host code on top of a pool: load on demand, eviction by the score of
 * Eq. 3, threshold prefetching ("Proactive Prefetching").  The paper gives neither weights nor
 * normalisation nor direction of Eq. 3 and no value of theta; this library reads them as follows.
 *   s_i = alpha * LRU_i + beta * freq_i + gamma * p_hat_i is a retention value: when the pool is out
 *   of pages the resident adapter with the LOWEST score is evicted first, equal scores by lowest id.
 *   LRU_i = k / (n - 1) where k is the adapter's position among the n residents ordered by the clock of
 *   their last request, oldest first (equal clocks by id; n = 1: LRU = 1).  freq_i = requests for i
 *   among the last `window` requests, divided by the largest such count among the residents (at
 *   least 1).  p_hat_i = the latest prediction handed over (0 before the first).  The clock counts
 *   requests.  The scores are evaluated in double precision, ((alpha*LRU) + (beta*freq)) + (gamma*p),
 *   once per load that finds the pool full; victims are then taken in that order until the load fits.
 *   Residents that plora_evict reports BUSY (their own copy is still running, or an open batch uses them)
 *   are passed over; if a load on demand finds nothing else to evict, the host waits for the copy of the
 *   lowest-scored such resident and evicts that one (the request could not be served before its own
 *   load anyway); a prefetch never waits.
 *   Prefetching: adapters with p_hat_i > theta that are not resident are loaded, most probable first
 *   (equal probabilities by id); room is made with the same score but only among residents with
 *   p_hat <= theta, and when none of those is left the remaining prefetches are dropped.
 * Every pointer is a host pointer.  Not thread safe.  The pool must outlive the manager, and adapters
 * the manager handles must not be loaded or evicted behind its back. */
typedef struct plora_manager plora_manager;
typedef struct {
  double alpha, beta, gamma; /* weights of Eq. 3, each >= 0 */
  double theta;              /* prefetch threshold on p_hat, 0 .. 1 */
  int32_t window;            /* requests the frequency term looks back over, >= 1 */
} plora_manager_config;
typedef struct {
  uint64_t hits, misses;       /* requests that found their adapter resident / not (cold starts) */
  uint64_t loads, evictions;   /* done by the manager */
  uint64_t failed_loads;       /* requests whose load found no room even after evictions */
  uint64_t skipped_busy;       /* victims passed over because plora_evict said BUSY */
  uint64_t waited_for_busy;    /* host waits for a busy victim's copy (loads on demand with nothing else to evict) */
  uint64_t prefetch_loads, useful_prefetches, wasted_prefetches; /* prefetched; requested before eviction; evicted unrequested */
  uint64_t prefetch_no_room;   /* prefetch rounds cut short for lack of unpredicted victims */
  /* memory utilisation (Sec. V-A lists it as a metric), sampled after every successful load once the pool
   * has first run out of pages: page_util = used pages / pages, byte_util = resident adapter bytes / pool bytes */
  uint64_t util_samples;
  double page_util_sum, page_util_min, byte_util_sum, byte_util_min;
} plora_manager_stats;

/* n_adapters: ids 0 .. n_adapters - 1 (at most the pool's max_adapters).  INVAL for values out of range. */
int plora_manager_create(plora_pool* pool, int32_t n_adapters, const plora_manager_config* config, plora_manager** out);
int plora_manager_destroy(plora_manager* manager);
/* What a load of adapter `id` needs: its rank, scale and page-locked host blob (NULL for a placement-only
 * pool), as plora_load_adapter takes them.  BUSY while the adapter is resident. */
int plora_manager_set_adapter(plora_manager* manager, int32_t id, int32_t rank, float scale, const void* pinned_host_ptr);
/* p_hat: n_adapters predicted access probabilities (copied), or NULL for "no prediction" (p_hat = 0). */
int plora_manager_set_prediction(plora_manager* manager, const float* p_hat);
/* One request for adapter `id`: advances the clock and the frequency window; a resident adapter is a hit
 * (*hit_out = 1); otherwise (*hit_out = 0) its load is started on copy_stream, after evictions by score if
 * the pool is full (failed_loads counts the case that no room could be made; the call still returns OK).
 * INVAL for an id that was not registered; errors of the pool are passed on. */
int plora_manager_request(plora_manager* manager, int32_t id, plora_stream copy_stream, int32_t* hit_out);
/* Takes the prediction for the coming interval and starts the loads it asks for on prefetch_stream (give
 * it a stream of its own, so that loads on demand do not queue behind them).  *n_started_out: loads started. */
int plora_manager_prefetch(plora_manager* manager, const float* p_hat, plora_stream prefetch_stream, int32_t* n_started_out);
/* Inspection.  Scores of the residents (ids ascending; at most cap entries written, *n_out = residents);
 * the residents alone; bit 0 = resident, bit 1 = prefetched and not requested since; the counters; the
 * decisions so far as (kind, id) pairs, kind 0 = load, 1 = evict (at most cap_pairs written, *n_pairs =
 * pairs recorded; clear != 0 empties the record). */
int plora_manager_scores(plora_manager* manager, int32_t* ids_out, double* scores_out, int32_t cap, int32_t* n_out);
int plora_manager_residents(plora_manager* manager, int32_t* ids_out, int32_t cap, int32_t* n_out);
int plora_manager_state(plora_manager* manager, int32_t id);
int plora_manager_get_stats(plora_manager* manager, plora_manager_stats* out);
int plora_manager_log(plora_manager* manager, int32_t* out, int64_t cap_pairs, int64_t* n_pairs, int32_t clear);

/* Page size from workload characteristics (the paper's discussion section names adaptive page sizes as
 * future work and says no more; Sec. III-C fixes only that an adapter of S bytes takes ceil(S / P) pages).
 * This library's reading: among the powers of two in [min_page, max_page], take the LARGEST page size whose
 * expected internal fragmentation,
 *     frag(P) = sum_k weight_k * (ceil(S_k / P) * P - S_k)  /  sum_k weight_k * ceil(S_k / P) * P ,
 * over the ranks the workload is expected to hold (S_k = bytes of a rank-ranks[k] adapter of this layout,
 * weight_k >= 0 its expected share of the resident adapters) stays at or below max_internal_frag: larger
 * pages mean fewer page-table entries per batch and fewer, longer copies per load, and the bound keeps what
 * they waste in check.  If no candidate meets the bound, the candidate with the smallest frag (the smaller
 * page on a tie).  Host only.  page_bytes_out / frag_out (may be NULL): the choice and its frag.
 * INVAL for n < 1, a rank < 1, a negative or all-zero weight vector, page bounds that are not powers of two
 * >= 4096 with min_page <= max_page, or a bound outside [0, 1). */
int plora_suggest_page_bytes(const plora_layout* layout, const int32_t* ranks, const double* weights, int32_t n,
                             double max_internal_frag, size_t min_page, size_t max_page, size_t* page_bytes_out,
                             double* frag_out);

/* Measurement aids for benchmarks; no part of the method (Sec. V-A asks for throughput and memory
 * figures, which want a roof measured on the same GPU beside the published peaks).
 * plora_probe_stream runs a bare kernel, 3 warm-up launches and then `iters` timed ones on `stream`,
 * in which every workgroup walks over tiles in turn: w_tile bytes of a w_bytes buffer read with
 * streaming 16-byte loads, then y_tile bytes of a y_bytes buffer read, changed and written back
 * (y_bytes = y_tile = 0: the plain streaming read).  One launch reads w_bytes, and reads and writes
 * (w_bytes / w_tile) * y_tile bytes of y (wrapping around y_bytes).  The buffers are allocated, filled
 * and freed inside the call, which synchronises the stream.  ms_per_launch: host.  INVAL unless the
 * tiles are multiples of 4096, w_tile >= 4096, and each buffer is a whole number of tiles of at most 2^36 bytes.
 * plora_probe_h2d times `iters` copies of one page-locked host buffer of `bytes` bytes (allocated
 * inside) to the device on `stream`, after one warm-up copy: the rate a single large pinned copy
 * reaches, to hold the adapter loads against. */
int plora_probe_stream(uint64_t w_bytes, uint64_t y_bytes, uint32_t w_tile, uint32_t y_tile, int32_t iters,
                       plora_stream stream, double* ms_per_launch);
int plora_probe_h2d(uint64_t bytes, int32_t iters, plora_stream stream, double* ms_per_copy);

/* ---------------------------------------------------------------------------------------------
 * Traffic predictor (Sec. III-A), host only: every pointer below is a host pointer and no call
 * touches the GPU.  A stack of `layers` LSTM layers of `hidden` units over a sliding window of
 * `window` prediction intervals, followed by a fully connected layer that gives one access
 * probability per adapter for the next interval (the paper: 2 layers, 64 units); trained with
 * Adam on Eq. 2 (binary cross-entropy summed over the adapters, averaged over a minibatch) from a
 * replay buffer of the most recent `replay` intervals (the paper: lr 1e-3, batch 64, 10,000
 * observations, an update every 100 requests).  An interval's input is the vector of its
 * normalised access counts c / (1 + c); the first layer's input weights are one row of 4 * hidden
 * values per adapter (its learned embedding).
 * Parameter vector, in this order: layer 0: E[n_adapters][4H], W_hh[4H][H], b[4H]; layers l > 0:
 * W_ih[4H][H], W_hh[4H][H], b[4H]; output: W_fc[n_adapters][H], b_fc[n_adapters]; gate order in 4H:
 * input, forget, cell candidate, output.  Arithmetic is fp32.  Not thread-safe. */
typedef struct plora_predictor plora_predictor;
typedef struct {
  int32_t n_adapters; /* >= 1 */
  int32_t window;     /* intervals the LSTM runs over, 1 .. 1024 */
  int32_t hidden;     /* 1 .. 1024 */
  int32_t layers;     /* 1 .. 8 */
  int32_t replay;     /* intervals kept for training, >= 2 */
  int32_t batch;      /* samples per Adam step of plora_predictor_train, >= 1 */
  float lr, beta1, beta2, eps;
  uint64_t seed;      /* parameter initialisation (uniform in +-1/sqrt(hidden), biases 0) and minibatch sampling */
} plora_predictor_config;

/* INVAL for a value out of range, NOMEM. */
int plora_predictor_create(const plora_predictor_config* config, plora_predictor** out);
int plora_predictor_destroy(plora_predictor* predictor);

/* One finished interval: the adapter ids of its requests (n_ids entries, repeats count).  It becomes
 * the newest entry of the history and of the replay buffer (the oldest leaves when `replay` is
 * exceeded).  INVAL for an id outside [0, n_adapters). */
int plora_predictor_observe(plora_predictor* predictor, const int32_t* ids, int32_t n_ids);

/* Intervals currently in the replay buffer. */
int64_t plora_predictor_observed(const plora_predictor* predictor);

/* p_hat[n_adapters]: predicted probability that each adapter is requested in the interval that
 * follows the newest observed one (intervals before the first observation count as empty). */
int plora_predictor_predict(plora_predictor* predictor, float* p_hat);

/* `steps` Adam updates, each on `batch` samples drawn (splitmix64 on seed and a running counter)
 * uniformly from the replay buffer: a sample is an interval as the target and the `window`
 * intervals before it as the input.  mean_loss_out (may be NULL): Eq. 2 averaged over the samples of
 * all steps.  Does nothing while fewer than 2 intervals have been observed. */
int plora_predictor_train(plora_predictor* predictor, int32_t steps, float* mean_loss_out);

/* One Adam update on the given samples: target_pos[k] in [1, observed) is the replay position
 * (0 = oldest) of sample k's target interval.  INVAL for a position out of range. */
int plora_predictor_train_batch(plora_predictor* predictor, const int32_t* target_pos, int32_t n_samples,
                                float* mean_loss_out);

/* Worker threads of plora_predictor_train / _train_batch (1 .. 64, default 1): the samples of a
 * minibatch are dealt to the workers in turn and their gradients added in worker order, so results are
 * reproducible for a given thread count (and differ between counts only by fp32 summation order). */
int plora_predictor_set_threads(plora_predictor* predictor, int32_t threads);

/* Inspection: number of parameters; copy them out / in (param_count floats). */
int64_t plora_predictor_param_count(const plora_predictor* predictor);
int plora_predictor_get_params(const plora_predictor* predictor, float* out);
int plora_predictor_set_params(plora_predictor* predictor, const float* in);

/* Loss (Eq. 2) and its gradient for one explicit sample: seq[window][n_adapters] feature vectors,
 * oldest first; target[n_adapters] of 0 / 1.  loss_out / grad_out (param_count floats) may be NULL.
 * Leaves parameters and Adam state alone. */
int plora_predictor_loss_grad(plora_predictor* predictor, const float* seq, const float* target, float* loss_out,
                              float* grad_out);

/* The last hipError_t seen by a call that returned PLORA_ERR_HIP (0 if none). */
int plora_last_hip(void);

/* Library version, major * 100 + minor. */
int plora_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PLORA_H */
