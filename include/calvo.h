/*
 * calvo.h - C ABI of the MI355X prefix-hit prefill path.
 *
 * The path is the part of the CALVO serving design that runs on one GPU and its
 * host: reusable KVCache blocks that already sit in local host DRAM (the
 * paper's L2 tier, Section 2.2) are loaded into a paged KV space in HBM (L1)
 * and the prefill of the not-yet-computed query tokens runs over them
 * (Section 3.1: each loading stage moves a block once its source is ready and
 * its destination is allocated, signals completion upward, and compute starts
 * as soon as the blocks it needs are resident).  Here residency is tracked per
 * transformer layer, so attention of layer l overlaps loading of layers l+1...
 *
 * Conventions
 *  - Every function returns a status (CALVO_OK == 0, errors negative) and never
 *    aborts or throws.  calvo_last_error() gives a thread-local message.
 *  - All argument validation happens on the host before any device work is
 *    queued: a call that fails with CALVO_EINVAL / CALVO_ENOMEM has written
 *    nothing.
 *  - "DEVICE" pointers are HIP device memory of the current device, "HOST"
 *    pointers ordinary host memory, "PINNED" page-locked host memory obtained
 *    from hipHostMalloc (or a framework's pinned allocator).  The library never
 *    frees, reallocates or keeps caller memory beyond what each call states.
 *  - Element type: CALVO_BF16 (2 bytes, upper half of an IEEE fp32) or
 *    CALVO_F32.  The ingest path moves bytes and does not interpret them.
 *
 * Layouts (B = block_tokens, Hkv = n_kv_heads, D = head_dim; C order)
 *    pool      [n_layers][pool_blocks][2][B][Hkv][D]   2 = K then V
 *    host KV   [n_layers][host blocks][2][B][Hkv][D]   one layer every host_layer_stride bytes
 *    q, out    [total suffix tokens][Hq][D]            requests concatenated, see cu_suffix
 *    k_suffix, v_suffix  [total suffix tokens][Hkv][D]
 * The paper names blocks, tiers and the context/query split but no block size,
 * layout or precision; these are this library's definitions.
 *
 * Threads: one thread at a time per context (the library's own loader thread
 * aside); different contexts are independent.
 *
 * Environment (for tests and tuning; results stay within the stated tolerance
 * whatever they are set to).  Read by calvo_create: CALVO_ATTN_SPLITS = n
 * cuts every attention tile's context into n pieces; CALVO_SPLIT_MIN,
 * CALVO_SPLIT_FILL = parameters of the automatic cut (shortest piece, cost of
 * a workgroup's start and end, both in 32-key steps); CALVO_SCATTER_GRID =
 * workgroups of the zero-copy scatter; CALVO_MERGE_MIB = most bytes of
 * consecutive small layers that one transfer carries (default 256, 0 = every
 * layer by itself).  Read by every calvo_prefill_attn:
 * CALVO_ATTN_VARIANT = 3 or 4 forces the 8-wave or the 4-wave bf16 kernel.
 * Test hooks, read by calvo_create: CALVO_INGEST_DELAY_US = n makes the host
 * sleep n microseconds before it queues each transfer of the L2 -> L1 stage
 * (the loading stage becomes the slow one; nothing on the device changes);
 * CALVO_TEST_SCATTER_DELAY_US = n puts a bounded delay kernel of n microseconds
 * in front of every staged scatter (the scatter becomes the slow stage, so the
 * reuse of the staging ring is exercised against its worst timing);
 * CALVO_TEST_L3_FAIL_CHUNK = k makes the L3 loader report a failure instead of
 * moving its chunk number k (error handling can then be tested without a fault).
 */
#ifndef CALVO_H
#define CALVO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct calvo_ctx calvo_ctx; /* opaque: streams, staging buffers, per-layer events, table cache */

enum { CALVO_OK = 0, CALVO_EINVAL = -1, CALVO_ENOMEM = -2, CALVO_EHIP = -3, CALVO_ENOTREADY = -4 };
enum { CALVO_BF16 = 0, CALVO_F32 = 1 };
enum { CALVO_EV_QUERY = 0, CALVO_EV_HOST_WAIT = 1, CALVO_EV_STREAM_WAIT = 2 };

typedef struct {
  int32_t n_layers;
  int32_t n_q_heads;     /* multiple of n_kv_heads */
  int32_t n_kv_heads;
  int32_t head_dim;      /* multiple of 8, at most 256; the bf16 MFMA kernel needs 128 */
  int32_t block_tokens;  /* B; must be 16 */
  int32_t dtype;         /* CALVO_BF16 or CALVO_F32 */
  int64_t pool_blocks;   /* slots per layer */
  void*   pool;          /* DEVICE, caller-owned, 16-byte aligned; must outlive the context */
  size_t  staging_bytes; /* size of each device staging buffer (a whole number of blocks is used);
                            0 selects the zero-copy ingest: the scatter kernel reads the pinned
                            host blocks directly over PCIe and no staging buffer is allocated */
  int32_t n_staging;     /* number of staging buffers in the ring, 2..8 (0 = 2) */
  int32_t n_copy_streams;/* 0 or 1: one stream issues the host-to-device copies (one copy-engine stream
                            already fills the link; a second one has to share a hardware queue with the
                            compute stream and serialises loading with attention) */
  void*   compute_stream;/* hipStream_t the attention work is queued on, caller-owned;
                            NULL = the library creates and owns one */
} calvo_config;

/* One request: a reusable context of n_prefix_blocks whole blocks (already held in
 * host DRAM) followed by suffix_len tokens that are computed now (paper, Section
 * 2.2: static application context + dynamic user query). */
typedef struct {
  const void*    host_kv;            /* PINNED, caller-owned: block j of layer l starts at
                                        host_kv + l*host_layer_stride + j*block_bytes.  Must stay valid
                                        and unchanged until the last requested layer's event has fired. */
  int64_t        host_layer_stride;  /* bytes between consecutive layers */
  const int32_t* block_table;        /* HOST: n_prefix_blocks + ceil(suffix_len/B) slot ids in
                                        [0, pool_blocks), pairwise distinct; read during the call only */
  int32_t        n_prefix_blocks;    /* P / B */
  int32_t        first_ingest_block; /* blocks [0, first) are already resident in the pool (a prefix run
                                        shared with an earlier request) and are not loaded; usually 0 */
  int32_t        suffix_len;         /* S >= 0 */
} calvo_request;

/* Create a context for one pool.  Allocates the staging ring, one event per layer and
 * the internal streams on the current device.  CALVO_EINVAL for a bad shape or NULL pool,
 * CALVO_ENOMEM / CALVO_EHIP if a device resource cannot be obtained (nothing is leaked). */
int calvo_create(const calvo_config* cfg, calvo_ctx** out);

/* Waits for all work queued through the context, then releases what calvo_create made.
 * The pool and the caller's stream are left alone. */
int calvo_destroy(calvo_ctx* ctx);

/* L2 -> L1 loading stage (paper Section 3.1; footnote of Section 4.1: several concurrent
 * loads are needed to fill PCIe).  For every request r, layer l in [layer_begin, layer_end)
 * and prefix block j in [first_ingest_block, n_prefix_blocks):
 *     pool[l][block_table[j]]  <-  host block j of layer l        (raw bytes, bit exact)
 * No other pool byte is written.  Asynchronous: the call queues copy-engine transfers into
 * the staging ring and scatter kernels on internal streams, records layer l's event after
 * the last store of layer l, and returns.  Layers are issued in ascending order.  When the
 * loaded blocks of consecutive layers follow each other in host memory and several such
 * layers fit one staging buffer, up to 256 MiB of them cross PCIe as one transfer (every
 * transfer boundary costs link time): groups of 1, 2, 4 ... layers, shrinking again towards
 * layer_end so that the last layers travel alone; each layer keeps its own scatter and
 * event, which fires once its group has landed.
 * Errors (nothing queued): CALVO_EINVAL for NULL pointers, a layer range outside
 * [0, n_layers], slot ids outside the pool or repeated inside one request, negative counts,
 * first_ingest_block > n_prefix_blocks, a host_layer_stride smaller than the request's
 * blocks; CALVO_EHIP if HIP refuses a transfer (queued work so far still completes). */
int calvo_kv_ingest(calvo_ctx* ctx, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end);

/* Chunk-granular readiness (paper Section 3.1: a stage signals the stage above for every block it
 * has finished loading, so that the stage above can start on what has landed).  Same loads and same final pool bytes as calvo_kv_ingest; in addition layer l (entry
 * l - layer_begin of chunk_blocks, HOST array of layer_end - layer_begin entries) is loaded in chunks
 * of chunk_blocks block indices: chunk k = blocks [k*cb, (k+1)*cb) of every request's table, chunks in
 * ascending order, one event per chunk recorded after its last store.  When chunk k's event has fired,
 * blocks [0, (k+1)*cb) of every request are resident in layer l (a shared run occupies the same
 * indices in every table).  An entry of 0 loads that layer as a whole (no chunk events).  Entries
 * must be even (attention walks the context two blocks at a time) and non-negative.
 * calvo_prefill_attn on a layer loaded this way starts on each chunk's keys as soon as that chunk is
 * in - one launch per chunk over partial softmax results, merged at the end - instead of waiting for
 * the whole layer; its result is the same up to rounding.  Every transfer boundary costs PCIe time,
 * so chunks pay where the wait for a whole layer is exposed (the last layer of a load-bound
 * request, the first of a compute-bound one).  Errors as calvo_kv_ingest, plus CALVO_EINVAL for a
 * NULL or odd / negative chunk_blocks entry. */
int calvo_kv_ingest_chunked(calvo_ctx* ctx, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end,
                            const int32_t* chunk_blocks);

/* Number of chunks the most recent load of `layer` was cut into (0: loaded as a whole or never). */
int calvo_chunk_count(calvo_ctx* ctx, int layer, int* n_chunks);

/* The per-chunk signal: modes as calvo_layer_event.  CALVO_EINVAL if chunk is outside
 * [0, calvo_chunk_count(layer)). */
int calvo_chunk_event(calvo_ctx* ctx, int layer, int chunk, int mode, void* stream);

/* Three-stage loading: remote store (L3) -> local host DRAM (L2) -> HBM (L1), each stage moving a
 * block as soon as its source is ready and its destination is free, and signalling the stage above
 * (paper Section 3.1; Section 4.1 gives the L3 link as 400 Gbps).  The remote store is emulated:
 * the requests' host_kv may be ordinary pageable HOST memory; a loader thread owned by the context
 * copies it chunk by chunk with n_threads host threads into a ring of n_slots pinned buffers (the
 * bounded L2 staging area), never faster than l3_GBps, and hands every landed chunk to the L2 -> L1
 * stage of calvo_kv_ingest (copy engine into the device staging ring, scatter into the pool).  A ring
 * slot is reused once its host-to-device copy has finished.  Layer l's event is recorded after the
 * last chunk of layer l. */
typedef struct {
  size_t  chunk_bytes; /* bytes per pinned ring slot, rounded down to whole blocks and to the device
                          staging buffer size; 0 = the staging buffer size */
  int32_t n_slots;     /* pinned ring slots, 2..8 (0 = 3) */
  int32_t n_threads;   /* host threads of the L3 -> L2 copy, 1..32 (0 = 4) */
  double  l3_GBps;     /* emulated link rate in 1e9 bytes/s: a chunk of n bytes occupies the link for
                          at least n / rate; 0 = as fast as the host copies */
  int32_t chunk_ready; /* != 0: chunk-granular readiness as in calvo_kv_ingest_chunked with chunks of
                          chunk_bytes (an even number of blocks): the loader moves block indices
                          [k*cb, (k+1)*cb) of every request as chunk k and records its event when it is
                          queued for L2 -> L1; calvo_prefill_attn starts on each chunk as it lands */
  int32_t reserved;    /* 0 */
} calvo_l3_config;

typedef struct {
  int64_t bytes;        /* bytes moved L3 -> L2 */
  int32_t chunks;       /* ring slots filled */
  double  l3_busy_s;    /* time the emulated link was occupied (copy + throttle) */
  double  ring_wait_s;  /* time the loader waited for a free ring slot (L2 -> L1 slower than L3 -> L2) */
  double  total_s;      /* from the call to the last chunk handed to the L2 -> L1 stage */
} calvo_l3_stats;

/* Same result in the pool as calvo_kv_ingest (raw bytes, bit exact, nothing else written), with the
 * source in pageable host memory and the L3 -> L2 stage described above in front.  Returns after
 * validation and after starting the loader thread; loading proceeds in the background.  The source
 * memory must stay valid and unchanged until calvo_l3_wait (or the last layer's event).  A failure
 * inside the loader is returned once, by the first later call that depends on it (calvo_l3_wait, a
 * loading call, calvo_layer_event / calvo_prefill_attn on a layer it did not hand over); that call
 * also un-marks those layers, and the context can load again.  While a
 * loader runs, calvo_layer_event(QUERY) reports CALVO_ENOTREADY for layers not yet handed over,
 * HOST_WAIT / STREAM_WAIT and calvo_prefill_attn block the calling thread until the layer's last
 * chunk has been handed to the L2 -> L1 stage (the wait for L1 residency itself stays on the
 * device), and a further calvo_kv_ingest / calvo_kv_ingest_l3 call first waits for the loader.
 * Needs a context with staging buffers (staging_bytes > 0).  l3 == NULL selects all defaults.
 * Errors (nothing started): as calvo_kv_ingest, plus CALVO_EINVAL for out-of-range l3 fields or a
 * zero-copy context, CALVO_ENOMEM if the pinned ring cannot be allocated. */
int calvo_kv_ingest_l3(calvo_ctx* ctx, const calvo_request* reqs, int n_reqs, int layer_begin, int layer_end,
                       const calvo_l3_config* l3);

/* Blocks until the loader started by calvo_kv_ingest_l3 has handed over its last chunk (or failed)
 * and returns its status; stats (may be NULL) receives its counters.  CALVO_OK with zeroed stats if
 * no loader was started.  Device-side completion is still observed through calvo_layer_event. */
int calvo_l3_wait(calvo_ctx* ctx, calvo_l3_stats* stats);

/* Per-layer "blocks are resident" signal (paper Section 3.1: a stage signals the stage above
 * when a block has been loaded).  mode:
 *   CALVO_EV_QUERY        CALVO_OK if layer's ingest has finished, else CALVO_ENOTREADY
 *   CALVO_EV_HOST_WAIT    block the calling thread until it has
 *   CALVO_EV_STREAM_WAIT  make `stream` (a hipStream_t; NULL = the compute stream) wait for
 *                         it on the device; the host does not block
 * A layer that was never ingested through this context counts as ready.  The signal of a layer
 * belongs to the most recent loading call that covered the layer: to serve several requests through
 * one context, queue a request's calvo_prefill_attn calls (they capture the signal when they are
 * made) before the next request's loading call - its loading then runs while the first request still
 * computes - or the earlier request's attention waits for the later load as well. */
int calvo_layer_event(calvo_ctx* ctx, int layer, int mode, void* stream);

/* Compute stage for one layer (paper Section 2.1 prefill over a reused prefix; Section 3.1:
 * launched once the needed blocks are resident).  Queued on the compute stream, after a
 * device-side wait on layer's ingest event:
 *   1. if k_suffix/v_suffix are non-NULL, the suffix tokens' K and V are written to the
 *      request's suffix slots (token i of request r at absolute position P_r + i);
 *   2. out[i][h][:] = sum_t softmax_t(scale * <q[i][h], K[t][g]>) V[t][g],  t = 0 .. P_r + i,
 *      g = h / (Hq/Hkv), K/V fetched through the block table.
 * q, k_suffix, v_suffix, out: DEVICE, 16-byte aligned, layouts above, element type = dtype
 * (accumulation is fp32; bf16 output is rounded to nearest even).  cu_suffix: HOST,
 * n_reqs+1 ascending offsets into the token dimension, cu_suffix[0] == 0 and
 * cu_suffix[r+1]-cu_suffix[r] == reqs[r].suffix_len.  scale <= 0 selects 1/sqrt(D).
 * Block tables are copied during the call.  Tokens stored after position P+S-1 in the last
 * slot are never read.  Returns CALVO_EINVAL (nothing queued) on NULL / misaligned pointers,
 * inconsistent cu_suffix, bad layer or bad slot ids. */
int calvo_prefill_attn(calvo_ctx* ctx, int layer, const void* q, const void* k_suffix, const void* v_suffix,
                       void* out, const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, float scale);

/* A batch prepared once for all its layers.  calvo_prefill_attn validates the requests, plans the launch
 * and describes it to the device on every call; a prefill runs the same batch through every layer, so
 * calvo_batch_prepare does all of that once: it checks reqs / cu_suffix as calvo_prefill_attn does,
 * copies the block tables, decides the launch (kernel, tiles, split-KV pieces) and uploads the
 * descriptors to a device buffer of its own (queued on the compute stream).  calvo_prefill_attn_batch
 * then only queues the layer's work - the wait for the layer's blocks, the suffix append, the
 * attention - with the result of calvo_prefill_attn for the same arguments.  Several batches can be
 * alive and queued at once (each has its own descriptors).  A layer that was loaded in chunks gets its
 * chunk-following launches planned the first time that chunking is seen and kept with the batch.
 * calvo_batch_destroy waits for the compute stream (launches may still read the descriptors) and
 * frees the batch - its descriptor buffers go back to the context, which hands them to later batches
 * and frees them in calvo_destroy; it must precede calvo_destroy of its context.  Errors: as calvo_prefill_attn; CALVO_ENOMEM / CALVO_EHIP if the
 * descriptor buffers cannot be had (nothing is leaked). */
typedef struct calvo_batch calvo_batch;
int calvo_batch_prepare(calvo_ctx* ctx, const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, calvo_batch** out);
int calvo_batch_destroy(calvo_batch* batch);
int calvo_prefill_attn_batch(calvo_ctx* ctx, calvo_batch* batch, int layer, const void* q, const void* k_suffix,
                             const void* v_suffix, void* out, float scale);

/* The same operation for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments, result and errors are
 * those of calvo_prefill_attn; the call itself allocates nothing (no hipMalloc / hipFree / pinned
 * allocation).  What calvo_prefill_attn keeps in buffers it grows on demand - the request
 * descriptors, work items and block tables the kernels read, and the partial results of tiles whose
 * context is cut into pieces - lives in one array of fixed size inside the library's device image
 * (35.5 MiB per GPU, held until the process ends; its address is looked up once per device by
 * calvo_create).  Limits: 262144 descriptor words (about 80000 table entries over the batch) and
 * 2048 partial-result slots (pieces x head groups x waves per workgroup); a batch beyond either gets
 * CALVO_ENOMEM with nothing queued - use calvo_prefill_attn for it (long layers loaded in chunks are
 * the usual case).  The array is shared by every call on the GPU, whatever the context: calls are
 * ordered by the compute stream they are queued on, and calls that overlap on one GPU from different
 * streams or contexts race.  Nothing in it needs to start at zero (every word a kernel reads was
 * written by the same call). */
int calvo_prefill_attn_noalloc(calvo_ctx* ctx, int layer, const void* q, const void* k_suffix, const void* v_suffix,
                               void* out, const calvo_request* reqs, int n_reqs, const int32_t* cu_suffix, float scale);

/* ---- Inter-request scheduling (paper Section 3.2; compared policies: Section 4.3).  Host code only.
 *
 * Cost model: a linear function of two variables fitted by offline profiling - loading latency linear in the
 * number of context tokens to load, computation latency linear in the number of query tokens:
 *     T_load = load_per_token_s * ctx_tokens + load_fixed_s      (0 when ctx_tokens == 0)
 *     T_comp = comp_per_token_s * query_tokens + comp_fixed_s    (0 when query_tokens == 0)
 * Policies order the queue by a priority, smaller first; ties go to the earlier arrival, then to the
 * lower index:
 *     CALVO_POLICY_FIFO    arrival time
 *     CALVO_POLICY_SJF     T_load + T_comp of the model                 (optimises average TTFT)
 *     CALVO_POLICY_SJF_PT  query_tokens, the number of tokens to prefill (the paper's SJF-PT)
 *     CALVO_POLICY_LSTF    slack LST = deadline - T_load - T_comp        (optimises SLO attainment)
 *     CALVO_POLICY_EDF     deadline
 * Service is non-preemptive. */
typedef struct {
  double load_per_token_s, load_fixed_s, comp_per_token_s, comp_fixed_s;
} calvo_cost_model;

typedef struct {
  double  arrival_s;    /* submission time */
  double  deadline_s;   /* absolute TTFT deadline (LSTF, EDF); ignored by the other policies */
  int64_t ctx_tokens;   /* context tokens whose KVCache must be loaded */
  int64_t query_tokens; /* tokens that must be computed */
} calvo_job;

enum { CALVO_POLICY_FIFO = 0, CALVO_POLICY_SJF = 1, CALVO_POLICY_SJF_PT = 2, CALVO_POLICY_LSTF = 3, CALVO_POLICY_EDF = 4 };

/* Least-squares line seconds = per_token_s * tokens + fixed_s through n >= 2 profiled samples (one
 * call for the loading component, one for the computation component).  CALVO_EINVAL for NULLs,
 * n < 2 or samples that all have the same token count. */
int calvo_cost_fit(const double* tokens, const double* seconds, int n, double* per_token_s, double* fixed_s);

/* T_load and T_comp of one job under the model. */
int calvo_cost_estimate(const calvo_cost_model* model, const calvo_job* job, double* load_s, double* comp_s);

/* The job to serve next at time `now`: among the jobs with done[i] == 0 (done may be NULL) and
 * arrival_s <= now, the one with the smallest priority; *out_index = -1 if none has arrived.
 * model may be NULL for policies that do not use it. */
int calvo_sched_pick(int policy, const calvo_cost_model* model, const calvo_job* jobs, const unsigned char* done, int n,
                     double now, int* out_index);

/* Replays a whole trace on one server.  load_s / comp_s: the time each job's loading and computation
 * actually take (HOST arrays of n; NULL = the model's estimates).  pipelined == 0: one job at a time,
 * load then compute.  pipelined == 1: loading and computation are separate stages (Section 3.1), a
 * job is taken when the loading stage is free and computes when its load has finished and the compute
 * stage is free, in loading order.  pipelined == 2: both stages serve their highest-priority ready
 * request (Section 3.1: every stage dispatches by priority): the loading stage picks among
 * the arrived jobs, the compute stage among the loaded ones, decisions in time order, the compute stage
 * first at equal times.  Whenever the (loading) stage is free and a job has arrived, the policy picks; if
 * none has arrived the server idles until the next arrival.  Outputs: start_s[i] (loading starts) and
 * finish_s[i] (first token; TTFT_i = finish_s[i] - arrival_s). */
int calvo_sched_simulate(int policy, const calvo_cost_model* model, const calvo_job* jobs, int n, const double* load_s,
                         const double* comp_s, int pipelined, double* start_s, double* finish_s);

/* ---- Slot allocation for the paged KV space with proactive reservation (paper Section 3.1:
 * when a lower-level transfer is issued, the destination space one level up is requested at the same
 * time, so a block can move on as soon as it arrives; its footnote: when HBM is short the scheme
 * falls back to allocating reactively, when space comes back).  Host code only; thread safe.  A slot carries a reference count: a
 * prefix run shared by several requests is referenced once per request and becomes free when the
 * last one releases it.  Which free slot a call hands out is unspecified (distinct, in range, free). */
typedef struct calvo_pool calvo_pool;

/* Bookkeeping for n_blocks slots (0 < n_blocks < 2^31), all free. */
int calvo_pool_create(int64_t n_blocks, calvo_pool** out);
int calvo_pool_destroy(calvo_pool* pool);

/* n distinct free slots -> slots[0..n) (HOST), each with one reference; all or nothing:
 * CALVO_ENOMEM (nothing reserved) if fewer than n are free. */
int calvo_pool_reserve(calvo_pool* pool, int32_t n, int32_t* slots);
/* One more reference on each listed slot; all must be in use (CALVO_EINVAL, nothing changed, otherwise). */
int calvo_pool_retain(calvo_pool* pool, const int32_t* slots, int32_t n);
/* Drops one reference per listed entry; a slot without references becomes free.  All or nothing:
 * CALVO_EINVAL if an entry is out of range or has no reference left. */
int calvo_pool_release(calvo_pool* pool, const int32_t* slots, int32_t n);
/* Any of the outputs may be NULL.  n_refs = sum of all reference counts. */
int calvo_pool_counts(calvo_pool* pool, int64_t* n_free, int64_t* n_used, int64_t* n_refs, int64_t* n_waiting);

/* Admission of a request, called when its lower-level transfer is issued (proactive allocation).
 * The request maps n_shared slots that are already in use (a prefix run it shares; distinct) and
 * needs n_own new ones.  If no earlier admission is waiting and n_own slots are free:
 * table[0..n_shared+n_own) = the shared slots (one more reference each) followed by the new slots,
 * CALVO_OK.  Otherwise (HBM short) the request joins the wait queue - reactive allocation -
 * *ticket identifies it and the call returns CALVO_ENOTREADY; its shared slots are referenced from
 * this moment so the run cannot be freed under it.  CALVO_ENOMEM if n_own exceeds the whole pool,
 * CALVO_EINVAL for bad arguments (nothing changed). */
int calvo_pool_admit(calvo_pool* pool, const int32_t* shared, int32_t n_shared, int32_t n_own, int32_t* table,
                     int64_t* ticket);
/* Reactive path: completes a queued admission if it is the oldest one waiting and its slots are free
 * now (table as above, CALVO_OK), else CALVO_ENOTREADY.  Queued admissions are served strictly in
 * arrival order.  CALVO_EINVAL for an unknown ticket. */
int calvo_pool_retry(calvo_pool* pool, int64_t ticket, int32_t* table);
/* Withdraws a queued admission and gives back its references on the shared run. */
int calvo_pool_cancel(calvo_pool* pool, int64_t ticket);

/* ---- The multi-request dispatcher (paper Section 3.1: each loading stage and the compute stage has a
 * dispatcher and an executor of its own and the stages run concurrently on different requests; a
 * block moves up one level only if it has arrived from the level below and its destination is
 * allocated; the destination is requested when the lower-level transfer is issued, and when HBM is
 * short the allocation is made reactively; Section 3.2: every stage serves its queue in the order of
 * the scheduling policy).
 *
 * The dispatcher owns one thread per stage:
 *   link   (three_stage != 0) L3 -> L2: takes the highest-priority submitted job, requests its HBM
 *          slots from `pool` (calvo_pool_admit) and streams its blocks, layer by layer in chunks, from
 *          the job's pageable host_kv through the pinned ring at no more than l3.l3_GBps;
 *   pcie   L2 -> L1: three_stage: takes the landed chunks in link order; a chunk moves on when it is in
 *          the ring and its job's slots are granted - a job the pool could not admit at once waits
 *          here (calvo_pool_retry, woken by calvo_dispatch_release), its chunks held in the ring and
 *          the link stalling behind them.  three_stage == 0: the jobs' host_kv is page-locked host
 *          memory, the stage picks the highest-priority job when the previous job's last block has
 *          landed, admits it (waiting here if HBM is short) and queues its layers;
 *   compute  takes the highest-priority job whose first layer has been handed over, and queues
 *          suffix append + attention of every layer on the compute stream, each behind the event of
 *          its layer's last block (a per-job event set: jobs loading at the same time do not share
 *          readiness state);
 *   done   waits for each job's last launch and stamps its first-token time.
 * A job's data: q, k_suffix, v_suffix, out are DEVICE arrays over all layers ([L][S][H][D], layer l at
 * l times the layer stride, 16-byte aligned); k_suffix / v_suffix may be NULL (suffix K/V already in
 * the pool).  host_kv / host_layer_stride as in calvo_request, for blocks
 * [n_shared, n_prefix_blocks).  Without a pool, block_table holds all n_prefix_blocks +
 * ceil(suffix_len/16) slots; with a pool it holds the n_shared slots of a run that is already resident
 * and in use, and the dispatcher obtains the rest.  All job memory stays valid until the job has
 * finished; block_table is copied by submit.  While a dispatcher is alive it is the only user of its
 * context.  With ctx == NULL the dispatcher is a dry run of the stage logic on the host clock: the
 * loading stage is busy sim_load_s per job, the compute stage sim_comp_s, with the same queues,
 * policy and admission; no device is touched. */
typedef struct calvo_dispatcher calvo_dispatcher;

typedef struct {
  int32_t policy;             /* CALVO_POLICY_*: the order every stage serves its queue in */
  int32_t three_stage;        /* != 0: emulated L3 link in front (pageable host_kv); 0: host_kv is pinned */
  calvo_cost_model model;     /* for SJF / LSTF priorities */
  calvo_l3_config l3;         /* three_stage: ring and link rate (chunk_ready is ignored) */
  calvo_pool* pool;           /* HOST, may be NULL: the caller assigns all slots itself */
} calvo_dispatch_config;

typedef struct {
  const void* host_kv;        /* HOST */
  int64_t host_layer_stride;
  const int32_t* block_table; /* HOST */
  int32_t n_prefix_blocks, n_shared, suffix_len, reserved;
  const void* q;              /* DEVICE */
  const void* k_suffix;       /* DEVICE or NULL */
  const void* v_suffix;       /* DEVICE or NULL */
  void* out;                  /* DEVICE */
  int64_t q_layer_stride;     /* bytes from layer l to layer l+1 of q; 0 = dense (suffix_len * Hq * D elements) */
  int64_t kv_layer_stride;    /* the same for k_suffix / v_suffix; 0 = dense (suffix_len * Hkv * D elements) */
  int64_t out_layer_stride;   /* the same for out; 0 = dense (suffix_len * Hq * D elements) */
  float scale;                /* <= 0: 1/sqrt(D) */
  float reserved2;
  double deadline_s;          /* TTFT deadline relative to submission (LSTF, EDF); <= 0: none */
  double sim_load_s, sim_comp_s; /* dry run only */
} calvo_dispatch_job;

typedef struct {              /* times in seconds since calvo_dispatch_create */
  double submit_s, load_start_s, load_end_s, compute_start_s, first_token_s;
  double alloc_wait_s;        /* time the job's blocks waited below for HBM slots (reactive allocation) */
  int32_t reactive;           /* != 0: the pool could not grant the slots when the transfer was issued */
  int32_t status;             /* CALVO_OK or the error that stopped the job */
} calvo_dispatch_result;

typedef struct {
  double  link_busy_s;        /* three_stage: time the emulated link was occupied (copy + throttle) */
  double  link_span_s;        /* from its first chunk's start to its last chunk's end */
  double  ring_wait_s;        /* time the link waited for a free ring slot */
  int64_t bytes;              /* bytes moved over the link */
  int64_t jobs_submitted, jobs_done;
} calvo_dispatch_stats;

/* Starts the stage threads.  ctx needs staging buffers.  CALVO_EINVAL for bad config fields,
 * CALVO_ENOMEM / CALVO_EHIP if the pinned ring or the threads cannot be had. */
int calvo_dispatch_create(calvo_ctx* ctx, const calvo_dispatch_config* cfg, calvo_dispatcher** out);
/* Queues a job; *id identifies it (ids count from 0 in submission order).  Returns at once.
 * CALVO_EINVAL (nothing queued) for bad counts or NULL pointers that the job needs, a host_kv that
 * is not page-locked in two-stage mode; CALVO_ENOMEM if the job can never fit the pool. */
int calvo_dispatch_submit(calvo_dispatcher* d, const calvo_dispatch_job* job, int64_t* id);
/* Blocks until the job's last attention launch has finished (its first token could be sampled) or the
 * job has failed; returns the job's status - calvo_last_error then holds what the failing call inside
 * the stage thread reported - and fills res (may be NULL). */
int calvo_dispatch_wait(calvo_dispatcher* d, int64_t id, calvo_dispatch_result* res);
/* The same without blocking: CALVO_ENOTREADY while the job is under way (res holds what is known). */
int calvo_dispatch_poll(calvo_dispatcher* d, int64_t id, calvo_dispatch_result* res);
/* The job's block table (shared run, then its own slots): *n entries into table[0..capacity).
 * CALVO_ENOTREADY before the slots are granted, CALVO_ENOMEM if capacity is too small (*n is set). */
int calvo_dispatch_table(calvo_dispatcher* d, int64_t id, int32_t* table, int32_t capacity, int32_t* n);
/* The request has left the GPU (its decode is over): gives its slots back to the pool - one reference
 * per table entry - and wakes the jobs that wait for slots.  Only after the job has finished
 * (CALVO_ENOTREADY before), once per job.  Jobs that wait for HBM make progress only through this
 * call: a caller that uses a pool smaller than its working set must release finished jobs. */
int calvo_dispatch_release(calvo_dispatcher* d, int64_t id);
int calvo_dispatch_stats_get(calvo_dispatcher* d, calvo_dispatch_stats* stats);
/* Waits for every submitted job to finish - finished jobs that were not released are released by this
 * call, so jobs that wait for their slots go on; jobs that still wait for slots when nothing else is
 * left to finish (the slots are held outside the dispatcher) are failed with CALVO_ENOMEM - stops the
 * threads, waits for the streams and frees the dispatcher.  Must precede calvo_destroy. */
int calvo_dispatch_destroy(calvo_dispatcher* d);

/* Measurement helper: duration in milliseconds of the most recent attention kernel queued by
 * calvo_prefill_attn for `layer` (HIP events recorded around the kernel on the compute
 * stream).  Blocks until that kernel has finished.  CALVO_ENOTREADY if none was queued. */
int calvo_attn_kernel_ms(calvo_ctx* ctx, int layer, float* ms);

/* Planning helper (host code, needs no GPU; host_kv is only used as an address): how
 * calvo_kv_ingest / calvo_kv_ingest_chunked would move layers [layer_begin, layer_end) of these
 * requests across PCIe with staging buffers of staging_blocks blocks of block_bytes bytes (0 = the
 * zero-copy mode) and at most merge_bytes per shared transfer (the library's default is 256 MiB).
 * chunk_blocks: NULL, or layer_end - layer_begin chunk sizes as for calvo_kv_ingest_chunked.
 * Outputs, HOST arrays of layer_end - layer_begin int32, either may be NULL:
 * transfer_of_layer[i] = index of the whole-layer transfer group that carries layer layer_begin + i
 * (layers with the same index share one transfer; -1 for a layer loaded in chunks), runs_of_layer[i] =
 * number of runs of consecutive host blocks the layer consists of (each run is a transfer of its
 * own, cut further where it exceeds a staging buffer).  CALVO_EINVAL for bad arguments. */
int calvo_ingest_plan(const calvo_request* reqs, int32_t n_reqs, int32_t layer_begin, int32_t layer_end,
                      int64_t block_bytes, int64_t staging_blocks, int64_t merge_bytes, const int32_t* chunk_blocks,
                      int32_t* transfer_of_layer, int32_t* runs_of_layer);

/* Planning helper (host code, needs no GPU): what calvo_prefill_attn would launch for a bf16, head
 * dim 128 batch with these lengths on a device with n_cus compute units.  prefix_blocks / suffix_lens:
 * HOST arrays of n_reqs.  Outputs (any may be NULL): *kernel as in calvo_attn_kernel_info,
 * *tile_tokens = suffix tokens per work item, *pieces = split-KV pieces a tile's context is cut into at
 * most (1 = no cut; pieces are never shorter than 48 sub-tiles of 32 keys), *n_workgroups of the
 * launch.  The choice replays the launch on the device's workgroup slots and cuts tiles when that
 * shortens it: too few tiles for the chip (the paper's requests: long contexts with short queries), or a
 * workgroup count just above a whole number of rounds.  CALVO_EINVAL for bad arguments. */
int calvo_attn_plan(int32_t n_q_heads, int32_t n_kv_heads, int32_t n_cus, const int32_t* prefix_blocks,
                    const int32_t* suffix_lens, int32_t n_reqs, int32_t* kernel, int32_t* tile_tokens,
                    int32_t* pieces, int32_t* n_workgroups);

/* Planning helper (host code, needs no GPU): the work items of that launch, in launch order.  A work
 * item is one tile of tile_tokens suffix tokens of one request over a range of its context, counted
 * in sub-tiles of 32 keys; the pieces of a cut tile follow each other and partition [0, ceil(keys the
 * tile's last row sees / 32)).  chunk_blocks = 0: a layer loaded as a whole (pieces as calvo_attn_plan
 * says); chunk_blocks > 0 (even): a layer loaded with calvo_kv_ingest_chunked in chunks of that many
 * blocks - piece k of a tile then covers the sub-tiles of chunk k inside the request's prefix and
 * belongs to launch k, which waits for chunk k only; the rest of the tile is its last piece, in the
 * last launch, which waits for the whole layer.  items: HOST array of 6 * capacity int32, filled
 * with (request, tile, first sub-tile, end sub-tile, pieces of the tile, launch) per work item;
 * *n_items: their number.  CALVO_ENOMEM if capacity is too small (*n_items is set; items may be NULL
 * with capacity 0 to ask for the count), CALVO_EINVAL for bad arguments. */
int calvo_attn_plan_items(int32_t n_q_heads, int32_t n_kv_heads, int32_t n_cus, const int32_t* prefix_blocks,
                          const int32_t* suffix_lens, int32_t n_reqs, int32_t chunk_blocks, int32_t* items,
                          int32_t capacity, int32_t* n_items);

/* Measurement helper: which attention kernel the most recent calvo_prefill_attn for `layer` chose
 * (*kernel: 3 = 8-wave workgroups with 64-token tiles, 4 = two 4-wave workgroups per CU with 32-token
 * tiles, 0-2 = comparison variants, -1 = the vector-ALU kernel for fp32 pools / other head dims) and
 * how many workgroups its work items made (*n_workgroups; 0 for the vector-ALU kernel).  Either
 * output may be NULL.  CALVO_ENOTREADY if none was queued. */
int calvo_attn_kernel_info(calvo_ctx* ctx, int layer, int* kernel, int* n_workgroups);

/* Measurement helper: the rate the matrix pipes of the current device sustain on bf16 MFMAs alone
 * (shape = CALVO_MFMA_16x16x32, the shape of the attention kernels, or CALVO_MFMA_32x32x16; two waves
 * per SIMD on every CU, operands in registers), for the operand data the caller supplies: operands =
 * DEVICE, 16 KiB of bf16 values (the first 8 KiB feed the A operands, the rest the B operands); sink =
 * DEVICE, at least 512 * 4 bytes per compute unit, receives the accumulators.  Runs on the default
 * stream: one warm-up launch, then `repeats` launches of `iters` x 16 (32x32x16) or `iters` x 32
 * (16x16x32) MFMAs per wave - the same number of products; *tflops = the fastest of them, *ms (may be
 * NULL) its duration.  The published peak assumes the top clock; the sustained rate depends on how
 * much the operand bits toggle and on the shape.  CALVO_EINVAL for bad arguments, CALVO_EHIP if HIP
 * refuses. */
enum { CALVO_MFMA_16x16x32 = 0, CALVO_MFMA_32x32x16 = 1 };
int calvo_mfma_peak(const void* operands, void* sink, int iters, int repeats, int shape, double* tflops, double* ms);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* calvo_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CALVO_H */
