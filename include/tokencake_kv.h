/*
 * tokencake_kv — paged KV-cache offload / upload for one AMD MI355X (gfx950).
 *
 * The library implements the data path of the paper's Temporal Scheduler
 * (Sec. 4.1 runtime event loop; Sec. 6.3 "CPU Migration Infrastructure"):
 * while an agent waits on a function call its idle KV blocks are copied to
 * pinned CPU memory (offload), and before the call is predicted to finish they
 * are copied back into newly reserved GPU blocks and the agent's block table is
 * pointed at them (upload).  It also keeps the block bookkeeping that Sec. 6.3
 * describes: a GPU free list with reference counts and the pending-free rule,
 * and a CPU pool of fixed-size slots recycled through a free list.
 *
 * Layouts (the paper fixes none; sizes follow Sec. 7.6):
 *   planes      P = 2 * num_layers, plane p = 2*layer + kv   (kv: 0 = K, 1 = V)
 *   KV pool     DEVICE memory, pool[p][block][page_bytes]   (plane-major)
 *   scales      DEVICE memory or NULL, scales[s][block], 32-bit words,
 *               scales_per_block in {0, 1, P}
 *   host record rec = roundup256(P*page_bytes + 4*scales_per_block) bytes per block:
 *               [page 0 | ... | page P-1 | scale words | zero pad]
 *   host buffer HOST pinned memory, 16-B aligned, n consecutive records, record j = block ids[j]
 *
 * Conventions
 *   - every function returns TC_OK (0) or a negative TC_ERR_* code; nothing throws
 *     or aborts.  All validation happens before anything is enqueued or any state
 *     changes: an error return means the call had no effect.  No C++ exception
 *     leaves the library; the process running out of host memory inside a call is
 *     reported as TC_ERR_HOST_NOMEM.
 *   - id arrays are HOST pointers (int32) and are copied before the call returns.
 *   - tc_offload / tc_upload are asynchronous: they return after enqueueing on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream).  Work
 *     later enqueued on the same stream is ordered after them; the host buffer /
 *     the pool may be read once the stream (or tc_sync) has completed.  Transfers
 *     of one context that touch the same blocks or the same arena allocation are
 *     ordered among themselves even when they are put on different streams.
 *     Against anything else the library orders nothing: work the caller has in
 *     flight on other streams that writes the pool, a host buffer or a block
 *     table must be ordered before `stream` by the caller (event or synchronise).
 *   - the caller owns the pool, the scales, block tables and any host buffer not
 *     obtained from tc_host_alloc.  The context owns its staging ring and arena.
 *   - one context serves one GPU (the device current at tc_create); calls on one
 *     context are serialised by an internal mutex.
 */
#ifndef TOKENCAKE_KV_H
#define TOKENCAKE_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TC_OK 0
#define TC_ERR_INVAL (-1)      /* bad argument, unallocated block, over-release      */
#define TC_ERR_RANGE (-2)      /* block id < 0 or >= num_blocks                      */
#define TC_ERR_DUP (-3)        /* the same block id twice in one transfer            */
#define TC_ERR_SHARED (-4)     /* block has more than one owner and must not move    */
#define TC_ERR_NOMEM (-5)      /* not enough free GPU blocks (all-or-nothing)        */
#define TC_ERR_HOST_NOMEM (-6) /* pinned arena has no run of slots that fits; host OOM */
#define TC_ERR_NOT_PINNED (-7) /* host buffer is not pinned / device ptr is not device */
#define TC_ERR_HIP (-8)        /* a HIP runtime call failed                          */
#define TC_ERR_LIMIT (-9)      /* beyond the fixed capacity of tc_offload_noalloc    */

typedef struct tc_ctx tc_ctx;

typedef struct {
    void *kv_base;              /* DEVICE, 256-B aligned, 2*num_layers*num_blocks*page_bytes bytes */
    void *scales;               /* DEVICE or NULL, scales_per_block*num_blocks 32-bit words        */
    uint32_t num_layers;
    uint32_t num_blocks;
    uint32_t page_bytes;        /* block_size * kv_heads * head_dim * elem bytes; multiple of 16   */
    uint32_t block_size_tokens;
    uint32_t scales_per_block;  /* 0, 1 or 2*num_layers                                            */
} tc_pool_desc;

enum { TC_PATH_AUTO = 0, TC_PATH_DIRECT = 1, TC_PATH_DIRECT_IF_DUPLEX = 2, TC_PATH_STAGED = 3 };

typedef struct {
    uint64_t host_arena_bytes;  /* pinned arena, allocated once; 0 = none (caller brings buffers)  */
    uint64_t staging_bytes;     /* device staging ring in total; 0 = default (2 slots of 4 GiB, or of the
                                   whole pool's records if that is less; halved until it fits, down to
                                   64 MiB, where device memory is short): a transfer that fits a slot is
                                   one copy launch and one DMA                                      */
    uint32_t staging_slots;     /* ring depth, >= 1; 0 = default                                   */
    uint32_t max_grid;          /* cap on workgroups per gather/scatter launch; 0 = one per tile   */
    uint32_t direct_offload;    /* which path an offload takes: TC_PATH_AUTO (0, the default) = through device
                                   staging and the copy engine, except while an upload of this context is in
                                   flight, when it goes direct (kernel-driven D2H traffic overlaps with H2D
                                   traffic on the link, two DMAs take turns), and except below
                                   auto_direct_bytes; TC_PATH_DIRECT = the gather kernel writes the records
                                   straight into the pinned host buffer, no staging, no DMA;
                                   TC_PATH_DIRECT_IF_DUPLEX = direct only while an upload is in flight;
                                   TC_PATH_STAGED = always gather into device staging, then DMA           */
    uint32_t direct_upload;     /* TC_PATH_AUTO (0) and TC_PATH_DIRECT = the scatter kernel reads the records
                                   straight from the pinned host buffer (at the link rate on an idle GPU, the
                                   least disturbed next to memory-bound kernels, and one pass through HBM
                                   instead of three); TC_PATH_STAGED = DMA into device staging, then scatter.
                                   With TC_PATH_AUTO a host buffer the GPU cannot map falls back to staging;
                                   with TC_PATH_DIRECT it is TC_ERR_NOT_PINNED                              */
    uint32_t direct_grid;       /* workgroups of a direct gather / scatter, and of a chunk's host tail
                                   (host_tail_div); 0 = defaults (gather 6, scatter 16, tails 6 / 8)   */
    uint32_t host_tail_div;     /* staged path only: the last 1/N of every chunk's blocks is moved by a few
                                   workgroups of the same copy launch straight to / from the pinned buffer,
                                   using the link while it would otherwise wait for the kernel, and the DMA
                                   carries that much less.  0 = automatic (N = 64 for transfers of more than
                                   one chunk whose kernels run in line with their DMAs, see overlap_kernels;
                                   none otherwise), 1 = never, N >= 2 = that N.  Applies to chunks of at
                                   least N blocks whose tail lies in one host buffer.                      */
    uint64_t auto_direct_bytes; /* TC_PATH_AUTO: offloads below this many record bytes go direct as well (one
                                   kernel instead of kernel + DMA saves ~19 us on an otherwise idle GPU; next to
                                   memory-bound kernels the staged path is the faster one); 0 = no such rule   */
    uint32_t overlap_kernels;   /* staged path: 0 (the default) = kernels and DMAs of a transfer in line on the
                                   caller's stream.  1 = a transfer of more than one chunk runs its copy kernels
                                   on a stream of the context's own, ordered with the caller's stream by events
                                   both ways, so that the kernel of one chunk runs under the DMA of its neighbour;
                                   such a transfer starts with a short chunk of 32 MiB (an upload ends with it).
                                   Every DMA, the table rewrite and completion stay on the caller's stream.  Up to
                                   2 % faster on an otherwise idle GPU; if the runtime places that stream behind
                                   a stream of long kernels on the same hardware queue, much slower               */
    uint32_t reserved0;         /* must be 0 */
} tc_opts;

typedef struct {
    const int32_t *block_ids;   /* HOST, n ids: sources (offload) or destinations (upload)         */
    uint32_t n;
    void *host_buf;             /* HOST pinned, n records                                          */
    int32_t *block_table;       /* DEVICE or NULL, upload only: first table entry to rewrite       */
} tc_xfer_desc;

typedef struct {
    uint32_t gpu_blocks_total, gpu_blocks_free, gpu_blocks_used, gpu_blocks_pending_free, gpu_blocks_shared;
    uint32_t ops_in_flight;
    uint64_t host_slots_total, host_slots_used;
    uint64_t n_offloads, n_uploads;           /* calls (a batch counts once)                       */
    uint64_t blocks_offloaded, blocks_uploaded;
    uint64_t bytes_offloaded, bytes_uploaded; /* host-record bytes                                 */
    /* filled for retired transfers while profiling is on (tc_set_profiling) */
    uint64_t gather_launches, scatter_launches;
    uint64_t gather_bytes, scatter_bytes;     /* record bytes the timed launches moved one way     */
    double gather_ms, scatter_ms;             /* sum of per-launch durations from HIP events       */
    uint64_t direct_launches, direct_bytes;   /* direct gathers: bound by the host link, not by HBM */
    double direct_ms;
    uint64_t d2h_copies, h2d_copies;          /* timed DMA chunks (all copies of one chunk together) */
    uint64_t d2h_bytes, h2d_bytes;
    double d2h_ms, h2d_ms;                    /* event pairs on the stream around each chunk's DMAs */
    uint64_t transfers_failed;                /* transfer calls that returned TC_ERR_HIP after validation */
    uint64_t transfers_overlapped;            /* staged transfers whose kernels ran on the context's own stream */
} tc_stats_t;

/* ---- life cycle ------------------------------------------------------------------------- */
/* Binds a pool (Sec. 6.3: the block pool owns the GPU<->CPU mapping).  Allocates the staging
 * ring, the id rings and the pinned arena on the current device and warms them with one DMA pass;
 * `opts` may be NULL for defaults.  The pool and the scales stay the caller's and must outlive the
 * context.  TC_ERR_INVAL for a bad description (zero sizes, page_bytes not a multiple of 16,
 * misaligned base, scales_per_block not in {0, 1, 2*num_layers}, scales given xor announced, an option
 * out of range, num_blocks * 2*num_layers * ceil(page_bytes / 4 KiB) above 2^31 - 1), TC_ERR_NOT_PINNED when kv_base / scales are not device memory, TC_ERR_HOST_NOMEM /
 * TC_ERR_HIP when an allocation fails; *out is NULL on any error. */
int tc_create(const tc_pool_desc *pool, const tc_opts *opts, tc_ctx **out);
/* Waits for every transfer in flight, then frees what the context owns (staging, rings, arena:
 * pointers from tc_host_alloc die with it).  NULL is a no-op. */
int tc_destroy(tc_ctx *ctx);
/* Host bytes per block (Sec. 7.6: 48 layers x K,V x 8 x 128 x 16 tokens x 2 B = 3 MiB). */
uint64_t tc_record_bytes(const tc_ctx *ctx);
const char *tc_strerror(int code);

/* ---- GPU block bookkeeping (Sec. 6.3) --------------------------------------------------- */
/* Pops n ids off the LIFO free list (first hand-out is 0,1,2,...); reference count := 1.
 * TC_ERR_NOMEM and no change when fewer than n blocks are free. */
int tc_alloc(tc_ctx *ctx, uint32_t n, int32_t *out_ids /* HOST, n */);
/* Claims exactly these ids (Sec. 6.3: an upload may take its original GPU blocks again); all-or-nothing.
 * TC_ERR_RANGE / TC_ERR_DUP for bad lists, TC_ERR_NOMEM when one of them is held or pending-free. */
int tc_alloc_at(tc_ctx *ctx, const int32_t *ids, uint32_t n);
/* Sec. 6.3: an upload takes its original GPU block again where it still can.  n blocks, all or nothing
 * (TC_ERR_NOMEM, nothing taken): out_ids[i] = preferred[i] wherever that block is still on the free
 * list, a fresh block from the head of the list otherwise.  Preferred blocks are claimed first, in
 * order, then the gaps are filled in order.  An id out of range, in use, pending-free or named
 * earlier in the call is simply no preference (so -1 means "any").  Finished transfers are retired
 * first.  preferred, out_ids: HOST, n entries each; they may be the same array. */
int tc_alloc_prefer(tc_ctx *ctx, const int32_t *preferred, uint32_t n, int32_t *out_ids);

/* One more owner for each id (shared prefix blocks).  TC_ERR_RANGE; TC_ERR_INVAL when an id is not
 * allocated.  No change on error. */
int tc_ref(tc_ctx *ctx, const int32_t *ids, uint32_t n);
/* Drops one owner per id.  At zero owners the block is free, unless a transfer touching it is
 * still in flight: then it is pending-free and becomes free when tc_poll / tc_sync retire that
 * transfer (Sec. 6.3: source blocks re-enter the free pool only once the copy is done). */
int tc_free(tc_ctx *ctx, const int32_t *ids, uint32_t n);
/* Copies the ids that have exactly one owner, order kept, into out_ids (HOST, room for n); *m = how
 * many.  TC_ERR_RANGE for a bad id. */
int tc_filter_private(tc_ctx *ctx, const int32_t *ids, uint32_t n, int32_t *out_ids, uint32_t *m);

/* ---- CPU block pool (Sec. 6.3: fixed-size blocks recycled, never returned to the OS) ----- */
/* n_blocks consecutive record slots from the pinned arena (first fit from the lowest address);
 * n_blocks = 0 gives NULL.  The memory stays the context's.  TC_ERR_HOST_NOMEM when no run of free
 * slots is long enough ("CPU capacity is insufficient", Sec. 4.2). */
int tc_host_alloc(tc_ctx *ctx, uint32_t n_blocks, void **host_buf);
/* host_buf must be a pointer tc_host_alloc returned (NULL is a no-op).  If a transfer using it
 * is in flight the slots are recycled when that transfer retires. */
int tc_host_free(tc_ctx *ctx, void *host_buf);

/* ---- transfers (Sec. 4.1, Sec. 6.3: issued asynchronously on a dedicated stream) --------- */
/* Offload: record j of host_buf <- block block_ids[j] (all planes, then scale words, then zero
 * pad).  Each block must be allocated and have exactly one owner (TC_ERR_INVAL / TC_ERR_SHARED);
 * ids must be distinct.  The pool and the block table are not written.  n = 0 is a no-op. */
int tc_offload(tc_ctx *ctx, const int32_t *block_ids, uint32_t n, void *host_buf, void *stream);
/* Upload: block new_block_ids[i] <- record i of host_buf, then block_table[i] = new_block_ids[i]
 * for i < n, written on `stream` after the data (Sec. 6.3: the upload puts the GPU mapping back).  block_table may
 * be NULL.  Same id rules as tc_offload. */
int tc_upload(tc_ctx *ctx, const void *host_buf, const int32_t *new_block_ids, uint32_t n,
              int32_t *block_table, void *stream);
/* Several agents in one call: their records share staging chunks and kernel launches, and the DMAs of
 * a chunk follow each other directly.  Prefer it to a run of single calls on the staged path: a DMA that
 * is enqueued behind a running one with a kernel in between is what the HIP runtime now and then carries
 * out at about half the link's rate (measured on MI355X), and a run of single staged transfers enqueues
 * every DMA but the first that way.  Ids must
 * be distinct across the whole batch; one bad descriptor fails the whole call with no effect.
 * Errors of all four transfer calls: TC_ERR_INVAL (NULL where data is expected, misaligned host
 * buffer, buffer longer than its arena allocation, unallocated block), TC_ERR_RANGE, TC_ERR_DUP,
 * TC_ERR_SHARED, TC_ERR_NOT_PINNED (host buffer not pinned, block table not device memory),
 * TC_ERR_HIP (a runtime call failed while enqueueing).  After TC_ERR_HIP the transfer must be treated as
 * failed and its destination (host records, or destination blocks and table entries) as undefined: part
 * of it may already be on the stream and still run.  Nothing that such work can read is reused early:
 * the transfer stays in flight, its blocks stay in flight (a tc_free on them gives pending-free), its
 * arena allocation and its span of device ids stay held, all until tc_poll / tc_sync retire it; if not
 * even its completion event could be recorded, the stream is drained inside the failing call instead. */
int tc_offload_batch(tc_ctx *ctx, const tc_xfer_desc *descs, uint32_t n_descs, void *stream);
int tc_upload_batch(tc_ctx *ctx, const tc_xfer_desc *descs, uint32_t n_descs, void *stream);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The same offload as tc_offload (record j of host_buf <- block block_ids[j],
 * gather_pages into a device staging chunk, then one D2H copy, all enqueued on `stream`), but with no
 * context: the staging chunk and the device copy of the ids live in a fixed device array that is part
 * of the library's code object (TC_NOALLOC_STAGING_BYTES + 4 KiB on every GPU the library is used on,
 * held until the process ends), and the call makes no hipMalloc / hipFree / event or heap allocation.
 *   pool       HOST pointer to the description (kv_base / scales are DEVICE memory, the caller's)
 *   block_ids  HOST, n distinct ids in [0, num_blocks); read before the call returns
 *   host_buf   HOST pinned, 16-B aligned, n records; valid once `stream` has completed
 * Limits: n <= TC_NOALLOC_MAX_BLOCKS and n * record bytes <= TC_NOALLOC_STAGING_BYTES, else TC_ERR_LIMIT
 * (a message on stderr says which).  Other errors as tc_offload (TC_ERR_INVAL, TC_ERR_RANGE, TC_ERR_DUP,
 * TC_ERR_NOT_PINNED, TC_ERR_HIP); an error means nothing was enqueued, except TC_ERR_HIP.
 * There is no bookkeeping: the caller keeps the blocks from being rewritten until `stream` completes.
 * All calls on one GPU share the one array, which keeps the previous call's bytes (nothing in it needs
 * clearing: each call writes all it reads): calls on the same stream are ordered, calls that overlap on
 * different streams of one GPU race and must be ordered by the caller. */
#define TC_NOALLOC_MAX_BLOCKS 1024u
#define TC_NOALLOC_STAGING_BYTES (64ull << 20)
int tc_offload_noalloc(const tc_pool_desc *pool, const int32_t *block_ids, uint32_t n, void *host_buf,
                       void *stream);

/* Retires completed transfers in issue order (pending-free -> free); never blocks. */
int tc_poll(tc_ctx *ctx);
/* Waits for every transfer issued so far, then retires them all. */
int tc_sync(tc_ctx *ctx);

/* ---- observation ------------------------------------------------------------------------ */
/* Snapshot of the counters (the part of the pressure snapshot of Sec. 3.2 that this layer owns:
 * free / used / pending-free / shared GPU blocks, CPU slots, transfer volume). */
int tc_stats(tc_ctx *ctx, tc_stats_t *out);
/* on != 0: bracket every gather / scatter launch with timing events on its stream. */
int tc_set_profiling(tc_ctx *ctx, int on);
/* The pinned arena (NULL / 0 without one). */
void *tc_arena_base(const tc_ctx *ctx);

/* ---- scheduling arithmetic around the copies (host only; Sec. 4.2, 4.3) ------------------ */
/* Transfer cost, Eq. 2: T_transfer(N) = (off_a + off_b*N) + (up_a + up_b*N), milliseconds. */
typedef struct {
    double off_a_ms, off_b_ms_per_block;
    double up_a_ms, up_b_ms_per_block;
} tc_cost_model;

/* A request in the waiting queue as Alg. 1 sees it. */
typedef struct {
    uint32_t kv_blocks;      /* incremental KV demand, in blocks              */
    double work_tokens;      /* total work, in tokens of decode throughput    */
} tc_waiting_req;

/* Least-squares fit of both lines from m >= 2 measurements (n_blocks[i], offload_ms[i], upload_ms[i]):
 * Eq. 2's per-block constants are meant to come from measurements on the target machine.  TC_ERR_INVAL
 * when m < 2 or all sizes are equal. */
int tc_cost_fit(const uint32_t *n_blocks, const double *offload_ms, const double *upload_ms, uint32_t m,
                tc_cost_model *out);
/* Measures the model on this context: for each size it claims that many free blocks and arena slots,
 * offloads them and uploads the same bytes back into the same blocks (`reps` times, median), so
 * the pool is unchanged afterwards.  Blocks on `stream` until done.  TC_ERR_NOMEM /
 * TC_ERR_HOST_NOMEM when the largest size does not fit. */
int tc_calibrate(tc_ctx *ctx, const uint32_t *sizes, uint32_t m, uint32_t reps, void *stream, tc_cost_model *out);
/* Eq. 2. */
double tc_estimate_transfer_ms(const tc_cost_model *model, uint32_t n_blocks);
/* Alg. 1 (ShouldOffload): 0 = reject, 1 = offload; *chosen = index of the first waiting request that
 * fits the freed blocks and the token capacity of the scheduling window, or -1.  Negative on bad
 * arguments. */
int tc_should_offload(const tc_cost_model *model, uint32_t req_blocks, double t_fc_ms,
                      double v_throughput_tokens_per_ms, const tc_waiting_req *queue, uint32_t n_queue,
                      int32_t *chosen);
/* Eq. 3: blocks this step may spend on uploads without touching what critical waiters need. */
uint32_t tc_upload_budget(uint32_t gpu_free, uint32_t d_critical, uint32_t shared_free);
/* Eq. 4: blocks to reserve for one candidate this step: min(remain, ceil(deficit / 2), budget). */
uint32_t tc_gradual_reserve(uint32_t remain, uint32_t deficit, uint32_t budget);

/* Sec. 4.2: four hard rejections come before any scoring of an offload: not enough CPU capacity,
 * a predicted stall no longer than the transfer, no waiting request that fits (Alg. 1), GPU memory
 * pressure under a configurable threshold.  They are tested in that order and the first that applies
 * is reported.  Pressure is gpu_used_blocks / gpu_total_blocks; "under" is strict. */
enum { TC_GATE_PASS = 0, TC_GATE_CPU_FULL = 1, TC_GATE_STALL_SHORT = 2, TC_GATE_NO_FIT = 3, TC_GATE_LOW_PRESSURE = 4 };
typedef struct {
    uint32_t req_blocks;        /* blocks the offload would free = CPU records it needs */
    uint32_t cpu_free_blocks;   /* free CPU records                                     */
    uint32_t gpu_used_blocks, gpu_total_blocks;
    double pressure_threshold;
    double t_fc_ms;             /* predicted stall                                      */
    double v_throughput_tokens_per_ms;
} tc_gate_input;
/* Returns 1 = none applies (*reason = TC_GATE_PASS, *chosen = the waiting request that fits),
 * 0 = rejected (*reason says why, *chosen = -1), TC_ERR_INVAL for NULL, NaN or gpu_total_blocks = 0.
 * chosen may be NULL.  The composite score that the paper applies afterwards has no published
 * weights and is not part of this library. */
int tc_offload_gate(const tc_cost_model *model, const tc_gate_input *in, const tc_waiting_req *queue,
                    uint32_t n_queue, int32_t *chosen, int *reason);

/* Sec. 4.3, one scheduling step of predictive upload: candidates are ranked by P_upload = I + U
 * (importance from the spatial scheduler's metric and urgency towards the predicted end of the call,
 * both supplied by the caller), the step's budget is Eq. 3, and each candidate in rank order reserves
 * Eq. 4's min(B_remain, ceil(B_deficit / 2), B_upload), B_remain shrinking as it goes.  Equal
 * P_upload: the more urgent candidate first, then the one listed first. */
typedef struct {
    double importance;   /* I */
    double urgency;      /* U */
    uint32_t deficit;    /* destination blocks this candidate still lacks */
} tc_upload_cand;
/* order[r] = index of the candidate of rank r; reserve[i] = blocks to reserve now for candidate i.
 * Both HOST arrays of n entries.  TC_ERR_INVAL for NULL or a NaN; nothing written then. */
int tc_upload_plan(const tc_upload_cand *cands, uint32_t n, uint32_t gpu_free, uint32_t d_critical,
                   uint32_t shared_free, uint32_t *order, uint32_t *reserve);

/* ---- request lifecycle and call-duration forecast (host only; Sec. 6.2, Sec. 4.1) -------- */
/* The five states of Sec. 6.2. */
enum { TC_RUNNING = 0, TC_PENDING_OFFLOAD = 1, TC_OFFLOADED = 2, TC_PENDING_UPLOAD = 3, TC_UPLOADED = 4 };
/* What drives them: the two endpoints and the scheduling loop. */
enum { TC_EV_CALL_START = 0, TC_EV_OFFLOAD_ISSUED = 1, TC_EV_OFFLOAD_DONE = 2, TC_EV_UPLOAD_ISSUED = 3,
       TC_EV_UPLOAD_DONE = 4, TC_EV_CALL_FINISH = 5 };
/* What the caller has to do after a step. */
enum { TC_ACT_NONE = 0, TC_ACT_RESUME = 1, TC_ACT_UPLOAD_NOW = 2, TC_ACT_WAIT = 3 };

typedef struct {
    uint8_t state;           /* TC_RUNNING ...                                          */
    uint8_t finish_seen;     /* call_finish arrived while the KV was away or in flight  */
    uint8_t copy_in_flight;  /* an offload or upload of this request has been issued    */
    uint8_t reserved;
} tc_req_state;

/* One transition.  Sec. 4.1: a request whose KV is already uploaded resumes at once on call_finish
 * (TC_ACT_RESUME); if the tool returns while the KV is on the CPU an immediate upload is due
 * (TC_ACT_UPLOAD_NOW); while a copy is in flight the finish is remembered (TC_ACT_WAIT) and acted
 * on when the copy completes.  TC_ERR_INVAL, and *req unchanged, for an event the state does not allow. */
int tc_lifecycle_step(tc_req_state *req, int event, int *action);

typedef struct tc_forecaster tc_forecaster;
/* Eq. 1 with weight alpha on the user's estimate; gamma is the weight of a new observation in the
 * moving average; default_ms is the system-wide constant used when nothing is known. */
int tc_forecaster_create(double alpha, double gamma, double default_ms, tc_forecaster **out);
int tc_forecaster_destroy(tc_forecaster *f);
/* Feeds the elapsed time that call_finish reports back into the type's moving average. */
int tc_forecaster_observe(tc_forecaster *f, uint32_t fn_type, double elapsed_ms);
/* Estimate for a type; has_user = 0 when the graph gives no predict_time. */
double tc_forecaster_estimate(const tc_forecaster *f, uint32_t fn_type, int has_user, double t_user_ms);

/* ---- residency map and CPU prefix-cache index (host only; Sec. 6.3) ---------------------- */
/* Sec. 6.3: the block pool owns the mapping between GPU blocks, CPU blocks and block hashes.  An
 * offload links the GPU block to its CPU record, marks it CPU-resident and enters its hash in a CPU
 * prefix-cache index; a lookup that hits there saves the recomputation but leaves an H2D transfer
 * entry that must complete before the request runs; the upload puts the GPU mapping back.  The paper
 * names neither the hash nor the index structure: keys are opaque 64-bit values here, and a lookup
 * answers for the longest leading run of keys present, since a block's key covers the prefix before
 * it.  The index stores addresses and ids only; it never touches the records or the pool, and it is
 * independent of any tc_ctx (the caller keeps it in step with its tc_offload / tc_upload calls).
 * All key and id arrays are HOST memory, read during the call.  Every call is all-or-nothing: on an
 * error the index is unchanged.  One internal mutex per index. */
typedef struct tc_index tc_index;
enum { TC_RES_ABSENT = 0, TC_RES_CPU = 1, TC_RES_H2D = 2 };
typedef struct {
    uint64_t key;
    void *cpu_record;   /* HOST address of the block's record (inside the buffer given at insert) */
    int32_t gpu_block;  /* TC_RES_CPU: the block it was offloaded from; TC_RES_H2D: where it is going */
    int32_t state;      /* TC_RES_CPU or TC_RES_H2D */
} tc_index_hit;

int tc_index_create(tc_index **out);            /* TC_ERR_INVAL for NULL, TC_ERR_HOST_NOMEM */
int tc_index_destroy(tc_index *ix);             /* NULL is fine */
/* After tc_offload(gpu_blocks, n, host_buf): key[j] -> record host_buf + j*record_bytes, CPU-resident,
 * remembered as coming from gpu_blocks[j].  TC_ERR_DUP if a key repeats or is already present. */
int tc_index_insert(tc_index *ix, const uint64_t *keys, const int32_t *gpu_blocks, void *host_buf,
                    uint64_t record_bytes, uint32_t n);
/* Prefix lookup: fills out[0..*hits) for the longest leading run of keys that are present. */
int tc_index_lookup(const tc_index *ix, const uint64_t *keys, uint32_t n, tc_index_hit *out /* n */,
                    uint32_t *hits);
/* A tc_upload into new_gpu_blocks has been issued for these keys: CPU-resident -> H2D transfer entry.
 * TC_ERR_INVAL unless every key is present and CPU-resident; TC_ERR_DUP for a repeated key. */
int tc_index_begin_upload(tc_index *ix, const uint64_t *keys, const int32_t *new_gpu_blocks, uint32_t n);
/* That upload has completed: the entries leave the index (the GPU holds the mapping again; the
 * caller may recycle the CPU records).  TC_ERR_INVAL unless every key is an H2D entry. */
int tc_index_finish_upload(tc_index *ix, const uint64_t *keys, uint32_t n);
/* Eviction of CPU-resident entries.  TC_ERR_INVAL if a key is absent or an upload is reading it. */
int tc_index_remove(tc_index *ix, const uint64_t *keys, uint32_t n);
/* How many of the keys are H2D entries: a request whose hits were uploaded may run when this is 0. */
uint32_t tc_index_pending(const tc_index *ix, const uint64_t *keys, uint32_t n);
uint64_t tc_index_size(const tc_index *ix);

/* Convenience keys (this library's choice, the paper gives none): 64-bit FNV-1a, and one key per
 * WHOLE block of token ids, each covering everything before it:
 *   key[i] = FNV1a( le64(key[i-1]) || le32(tokens[i*bs .. (i+1)*bs)) ),  key[-1] = parent.
 * A trailing partial block gets no key.  out needs n_tokens / block_size entries; *n_out = that count. */
#define TC_FNV_BASIS 0xCBF29CE484222325ull
uint64_t tc_fnv1a64(const void *data, uint64_t len, uint64_t basis);
int tc_chain_hashes(const int32_t *tokens, uint64_t n_tokens, uint32_t block_size, uint64_t parent,
                    uint64_t *out, uint64_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* TOKENCAKE_KV_H */
