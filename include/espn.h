/*
 * espn.h - C ABI of the MI355X (gfx950) re-ranking library.
 *
 * The library implements the re-ranking stage of multi-vector ("late interaction")
 * retrieval: for each query, the candidate documents named by a first-stage retriever
 * (Sec. 2.1; about a thousand per query, Sec. 4.4) are looked up in the token-embedding
 * table through per-document offsets (Sec. 4: the table's metadata is a list of offsets),
 * scored with the MaxSim operator (Eq. 1, Sec. 2.1) and ranked by score (Sec. 2.1).
 *
 * Conventions for every entry point
 *   - Plain C types only.  Every pointer argument says whether it is a HOST or a DEVICE
 *     pointer.  DEVICE pointers must belong to the device the table was loaded on.
 *   - `stream` is a hipStream_t passed as void* (NULL = the device's null stream).  Calls that
 *     take a stream only enqueue work on it and return; they never synchronise and never
 *     allocate or free device memory.
 *   - The return value is an espn_status.  Argument errors are found on the host before
 *     anything is enqueued.  Nothing throws or aborts across this boundary.
 *     espn_last_error() gives a message for the calling thread's last failure.
 *   - 16-bit embeddings are IEEE binary16 (Sec. 3.1: 16-bit vectors); products are accumulated
 *     in binary32; scores are binary32.  Inputs must be finite: the rank of a NaN score is
 *     unspecified.
 */
#ifndef ESPN_H
#define ESPN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum espn_status {
    ESPN_OK = 0,
    ESPN_ERR_ARG = 1,          /* null pointer, negative size, bad enum value */
    ESPN_ERR_SHAPE = 2,        /* sizes that contradict each other (k > K, workspace too small, ...) */
    ESPN_ERR_OFFSETS = 3,      /* offsets do not start at 0 or decrease somewhere */
    ESPN_ERR_ID_RANGE = 4,     /* a candidate id outside [0, n_docs) was met by a kernel */
    ESPN_ERR_NOMEM = 5,        /* host or device allocation failed */
    ESPN_ERR_HIP = 6,          /* a HIP runtime call failed; see espn_last_error() */
    ESPN_ERR_UNSUPPORTED = 7   /* a shape this build has no kernel for */
} espn_status;

typedef struct espn_table espn_table;   /* opaque; owned by the library */

/* Where the packed embedding rows live: in device memory; in pinned host memory, which the device can read
 * (either prefetch engine works); or in ordinary host memory, which only the host reads (espn_prefetch_packed
 * only: what a machine that refuses to pin a table of the paper's size still can do). */
enum { ESPN_RESIDENT_HBM = 0, ESPN_RESIDENT_HOST_PINNED = 1, ESPN_RESIDENT_HOST = 2 };

/* Static string for a status code. */
const char *espn_status_string(int status);

/* Message describing the calling thread's most recent failing call ("" if none). */
const char *espn_last_error(void);

/*
 * Register an embedding table (Sec. 3.1 / Sec. 4: token vectors per document plus offsets).
 *
 *   emb          [total_rows, dim] binary16, row-major, packed: document i owns rows
 *                offsets[i] .. offsets[i+1]-1.  DEVICE pointer if residency is
 *                ESPN_RESIDENT_HBM; pinned HOST pointer (hipHostMalloc) if
 *                ESPN_RESIDENT_HOST_PINNED; any HOST pointer if ESPN_RESIDENT_HOST.  BORROWED: never copied, never freed; the caller
 *                keeps it alive and unchanged until espn_table_free.  Must be 16-byte aligned.
 *   offsets_host [n_docs + 1] int64 HOST pointer, in rows; offsets[0] = 0, non-decreasing
 *                (a document may be empty).  COPIED (to the device); may be freed after the call.
 *   dim          vector length; a positive multiple of 8.  Multiples of 32 up to 256 run on the
 *                matrix-core kernel (32 and 128, the two the paper's models use, are the tuned
 *                ones), other values on a slower generic one.
 *   device       HIP device ordinal.
 *   out          receives the handle.
 *
 * Synchronous (copies the offsets and waits).  Errors: ARG, OFFSETS, NOMEM, HIP.
 */
int espn_table_load(const void *emb, const int64_t *offsets_host, int64_t n_docs, int32_t dim,
                    int32_t residency, int32_t device, espn_table **out);

/*
 * Register a compressed table (Sec. 6: 8-bit formats shrink the re-ranking index and with it the data
 * moved per query).  A token vector is stored as `dim` one-byte codes in the E4M3 format of the OCP
 * 8-bit floating point specification (no NaN codes allowed), and every document has one scale: a
 * stored component stands for doc_scale[doc] * decode(code).  Every entry point that takes a table
 * works on such a table; codes are widened exactly to binary16 inside the scoring kernel, products
 * accumulate in binary32 as for binary16 tables, and the scale multiplies the document's score.
 *
 *   codes           [total_rows, dim] uint8, row-major, packed like `emb` of espn_table_load; DEVICE or
 *                   pinned HOST pointer according to residency; BORROWED; 16-byte aligned.
 *   doc_scale_host  [n_docs] binary32 HOST pointer, each positive and finite; COPIED.
 *   dim             32 or 128 (ESPN_ERR_UNSUPPORTED otherwise); queries: 1..32 rows of binary16.
 * Other arguments and errors as espn_table_load.
 */
int espn_table_load_e4m3(const void *codes, const float *doc_scale_host, const int64_t *offsets_host,
                         int64_t n_docs, int32_t dim, int32_t residency, int32_t device, espn_table **out);

/* Release a table handle (the offsets copy and the library's own buffers; never `emb`).
 * Synchronises the device first.  NULL is allowed. */
int espn_table_free(espn_table *table);

/* Facts about a loaded table; any out pointer may be NULL. */
int espn_table_info(const espn_table *table, int64_t *n_docs, int64_t *total_rows, int32_t *dim,
                    int32_t *residency, int32_t *device);

/*
 * How the rows of the table are fetched by the scoring kernels:
 *   ESPN_FETCH_AUTO       decided per batch from what the library knows, nothing else: if espn_table_sample has
 *                         been called, cached if more than 5 % of the sampled pairs repeated a document, streaming
 *                         if not; before that, streaming for 64-byte rows, and for longer rows if the batch has at
 *                         most half as many (query, candidate) pairs as the table has documents.  The default.
 *   ESPN_FETCH_STREAMING  non-temporal loads: fastest when the queries of a batch list different documents
 *                         (uniformly drawn lists: 2 to 12 % faster than cached).
 *   ESPN_FETCH_CACHED     ordinary loads that leave the rows in the caches: fastest when the lists overlap,
 *                         whatever the batch size (lists drawn from a Zipf law: 10 to 36 % faster than streaming
 *                         from 64 queries per batch on).
 * The scores do not depend on it.  Takes effect from the next call on.  The same calls in the same order always
 * run the same kernels (no call looks at the clock, at a call count or at unfinished work).  Errors: ARG.
 */
enum { ESPN_FETCH_AUTO = 0, ESPN_FETCH_STREAMING = 1, ESPN_FETCH_CACHED = 2 };
int espn_table_set_fetch(espn_table *table, int32_t mode);

/*
 * Tell the library what this caller's candidate lists look like (Sec. 4.4: about a thousand candidates per query
 * from the first stage; popular documents recur): up to 4096 evenly spaced (query, candidate) pairs of the batch
 * are put into a hash set by one small kernel on `stream`, and the fraction whose document another sampled pair
 * had named already is kept with the table for ESPN_FETCH_AUTO (and espn_table_sharing_estimate).  Uniform lists
 * over 2 M documents give 0.002, Zipf(1.1) lists 0.3 and more.
 *
 * If the lists overlap (more than 5 % of the sampled pairs) and the table is in HBM with rows of 128 bytes or more
 * (64-byte rows were measured to gain nothing from what follows), the call also notes which
 * documents are popular: listed by at least two of the batch's queries and by at least one in 256 (counted over
 * the whole batch, one bit per document kept with the table; n_docs * 4 bytes of device memory are allocated and
 * freed inside the call).  From then on
 *   - launches that fetch through the caches do so for the popular documents only and stream the others past
 *     them, so that the popular ones stay there;
 *   - espn_rerank and espn_rerank_batches take batches of whole lists that fill the device many times over (a
 *     batch, or the batches of a queue that one launch scores together: at least three workgroups per compute
 *     unit, lists of up to 4096 candidates) in the order of their document ids:
 *     one more launch sorts a copy of every list by id, and the scoring launch walks all lists in that order at
 *     once, slice by slice, so that the queries that list a document ask for it at about the same time
 *     (2048 queries x 1000 Zipf candidates, 256-byte rows: 3.80 instead of 4.66 ms per batch).
 * Scores and ranks do not depend on any of this.  A later sample that finds no overlap switches it off again.
 *   cand  [B, K] int64, DEVICE.
 * SYNCHRONOUS: waits for `stream` (call it once when a workload starts, not per batch, and not while calls that
 * use the table are in flight on other streams).  Errors: ARG, HIP, NOMEM.
 */
int espn_table_sample(espn_table *table, const int64_t *cand, int32_t B, int32_t K, void *stream);

/* The result of the last espn_table_sample on this table, -1 if there was none.  estimate: HOST pointer.
 * Errors: ARG. */
int espn_table_sharing_estimate(const espn_table *table, float *estimate);

/*
 * MaxSim scores of every candidate (Eq. 1):
 *     scores[b,j] = sum over i < Q of  max over rows r of document cand[b,j] of  <q[b,i,:], emb[r,:]>
 * The candidate gather (offset lookup + streaming the document's rows) is fused into the
 * scoring kernel; no copy of the rows is made.
 *
 *   q       [B, Q, dim] binary16, DEVICE, 16-byte aligned.
 *   cand    [B, K] int64 document ids, DEVICE.
 *   scores  [B, K] binary32, DEVICE, written.
 *   Q       1 .. 64 on the matrix-core kernel (1 .. 32 for rows of more than 128 components); the
 *           generic kernel takes any Q with Q * dim * 2 bytes <= 64 KiB.
 * An empty document scores -infinity (empty max).  An id outside [0, n_docs) scores
 * -infinity and raises the table's error flag (see espn_table_check); nothing is read for it.
 * B = 0 or K = 0 is a no-op.  The table must be HBM-resident (ESPN_ERR_UNSUPPORTED otherwise).
 * One call takes up to 2^31 - 1 (query, candidate) pairs (ESPN_ERR_UNSUPPORTED beyond).
 * Errors: ARG, SHAPE, UNSUPPORTED, HIP.
 */
int espn_score(espn_table *table, const void *q, const int64_t *cand,
               int32_t B, int32_t Q, int32_t K, float *scores, void *stream);

/*
 * Ranked top-k of scored candidates (Sec. 2.1: sort by score): per query the k best of K in the
 * order (score descending, then document id ascending), best first.
 *
 *   scores      [B, K] binary32, DEVICE.        cand        [B, K] int64, DEVICE.
 *   out_ids     [B, k] int64, DEVICE, written.  out_scores  [B, k] binary32, DEVICE, written.
 *   0 <= k <= K.
 * Errors: ARG, SHAPE, HIP.
 */
int espn_topk(const float *scores, const int64_t *cand, int32_t B, int32_t K, int32_t k,
              int64_t *out_ids, float *out_scores, void *stream);

/* Bytes of DEVICE workspace espn_rerank needs for a batch of B queries with K candidates each: the scores
 * (4 bytes per pair, at the start), then room for the lists in id order (8 bytes per pair; see espn_table_sample),
 * each rounded up to 256 bytes. */
size_t espn_workspace_bytes(int32_t B, int32_t K);

/*
 * The whole hot path for an HBM-resident table: gather + MaxSim + ranked top-k.
 * Same result as espn_score into the workspace followed by espn_topk, both on `stream`; short candidate
 * lists are scored and ranked by one launch (espn_rerank_plan).
 *
 *   workspace        DEVICE, 256-byte aligned, at least espn_workspace_bytes(B, K) bytes; scratch
 *                    owned by the caller, contents undefined afterwards (it holds all B*K scores).
 * Errors: ARG, SHAPE, UNSUPPORTED, HIP.
 */
int espn_rerank(espn_table *table, const void *q, const int64_t *cand,
                int32_t B, int32_t Q, int32_t K, int32_t k,
                int64_t *out_ids, float *out_scores,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * The whole hot path for a QUEUE of batches of one shape (Sec. 5.4, 5.5: throughput under batched queries): the
 * same results as n_batches calls of espn_rerank, bit for bit, at the cost of a long launch instead of many short
 * ones.  Small batches (64 queries x 1000 candidates at dim 32: a 31 us scoring launch, of which the launch gap and
 * the two dependent look-ups at its start are a sixth, plus a ranking launch) are scored up to 16 at a time by ONE
 * launch that streams like one large batch, and ranked by one more; these chunks - or, for batches that fill the
 * device many times over by themselves, the batches - are dealt in turn to ESPN_BATCH_LANES streams of the library's
 * own (created with the table, default priority), so that the ranking of one chunk and the start of the next
 * overlap with the streaming of the one before.  The library's streams wait for everything enqueued on `stream`
 * before the call (nothing, if it is idle), and `stream` waits for all of the call's batches: to the caller it is
 * one asynchronous operation on `stream`, results valid when it is through.  The call may be captured into a HIP
 * graph (the hand-over to the library's streams and back becomes graph edges).
 *
 *   q, cand, out_ids, out_scores  HOST arrays of n_batches DEVICE pointers, each as in espn_rerank; the arrays
 *                                 themselves are read before the call returns.
 *   workspace                     DEVICE, 256-byte aligned, espn_batches_workspace_bytes(table, n_batches, B, Q, K, k)
 *                                 bytes (up to 3 x 16 x espn_workspace_bytes(B, K)); contents undefined afterwards,
 *                                 except that a call with n_batches <= ESPN_BATCH_LANES leaves the B*K scores of
 *                                 batch 0 at its start.
 * A queue that makes one launch runs on `stream` itself.  Not to be called for one table from several host
 * threads at once.
 * Errors: ARG, SHAPE, UNSUPPORTED, HIP (all argument checks are done before anything is enqueued).
 */
#define ESPN_BATCH_LANES 3
size_t espn_batches_workspace_bytes(const espn_table *table, int32_t n_batches, int32_t B, int32_t Q, int32_t K, int32_t k);

/*
 * How espn_rerank_batches would run a queue of this shape: `fuse` batches per scoring launch at most (the queue is
 * cut into `launches` chunks whose sizes differ by one at most), dealt to `streams` streams (1: the caller's own),
 * and the profiler names of the kernels of one chunk, separated by ';' (kernels: HOST, 256 bytes always suffice;
 * may be NULL, as any other out pointer).  Host arithmetic only.  Errors: ARG, SHAPE.
 */
int espn_batches_plan(const espn_table *table, int32_t n_batches, int32_t B, int32_t Q, int32_t K, int32_t k,
                      int32_t *fuse, int32_t *launches, int32_t *streams, char *kernels, size_t kernels_len);
int espn_rerank_batches(espn_table *table, int32_t n_batches, const void *const *q, const int64_t *const *cand,
                        int32_t B, int32_t Q, int32_t K, int32_t k,
                        int64_t *const *out_ids, float *const *out_scores,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * espn_rerank for callers that cannot allocate device memory and have no workspace to hand in: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  The B*K scores that espn_rerank keeps
 * in the caller's workspace go to a fixed array inside the library's code object instead (one copy per device,
 * sizeof(float) * ESPN_NOALLOC_MAX_PAIRS bytes, held until the process ends); its address on the table's device
 * was looked up when the table was loaded.  The call allocates and frees nothing, on the host or on the device.
 *
 *   Arguments and results as espn_rerank (same scoring and ranking kernels, same bits; the array has no room for
 *   lists in id order, so they are always scored as they come); B * K <= ESPN_NOALLOC_MAX_PAIRS, ESPN_ERR_SHAPE
 *   beyond.
 * All calls on one device share the array, whatever table or stream they name: two calls whose kernels may
 * overlap in time (different streams, or different host threads) race on it and must be ordered by the caller;
 * calls on one stream are ordered already.  Afterwards the array holds the scores of the last call.
 * Errors: ARG, SHAPE, UNSUPPORTED, HIP.
 */
#define ESPN_NOALLOC_MAX_PAIRS (4 * 1024 * 1024)
int espn_rerank_noalloc(espn_table *table, const void *q, const int64_t *cand,
                        int32_t B, int32_t Q, int32_t K, int32_t k,
                        int64_t *out_ids, float *out_scores, void *stream);

/*
 * How espn_rerank (and its variants) would run a batch of this shape on this table: the candidate list
 * of a query is cut into `slices` runs of `slice` candidates, one workgroup each; `launches` is 1 if the
 * scoring kernel also ranks (one slice of at most 256 candidates per query), 2 if the stand-alone ranking kernel
 * follows it, 3 if espn_rerank also sorts the lists by document id first (espn_table_sample; the variants for
 * partial re-ranking and a prior never do), 0 for an empty batch.  Host arithmetic only; any out pointer may be NULL.
 * For partial re-ranking pass K = R and k = min(k, R).  Errors: ARG, SHAPE.
 */
int espn_rerank_plan(const espn_table *table, int32_t B, int32_t Q, int32_t K, int32_t k,
                     int32_t *slices, int32_t *slice, int32_t *launches);

/*
 * The kernels espn_rerank would launch for a batch of this shape, by the names a profiler prints for them (template
 * arguments included), separated by ';': the scoring kernel, then the kernel that sorts the lists by document id
 * if one runs ahead of it (espn_table_sample), then the ranking kernel if a launch of its own ranks.
 * Lets a benchmark tie a counter profile to the kernels that actually run.  Empty for an empty batch.
 *   buf  HOST, buf_len bytes (256 always suffice); receives a NUL-terminated string.
 * Host arithmetic only.  Errors: ARG, SHAPE (k > K, or buf too small).
 */
int espn_rerank_plan_kernels(const espn_table *table, int32_t B, int32_t Q, int32_t K, int32_t k,
                             char *buf, size_t buf_len);

/*
 * Partial re-ranking (Sec. 4.4): the candidate list of a query arrives best-first from the first
 * stage; only its first R entries are scored with MaxSim and ranked, the remaining K - R entries
 * follow them in the order they came.  Writes the first k entries of that combined list.
 *
 *   cand        [B, K] int64, DEVICE.   0 <= R <= K,  0 <= k <= K.
 *   out_ids     [B, k] int64, DEVICE.   out_scores [B, k] binary32, DEVICE: the MaxSim score for
 *               ranks below R, NaN (not scored) from rank R on.
 *   workspace   DEVICE, 256-byte aligned, at least espn_workspace_bytes(B, R) bytes.
 * Only R documents per query are read from the table.  HBM-resident tables only.
 * Errors: ARG, SHAPE, UNSUPPORTED, HIP.
 */
int espn_rerank_partial(espn_table *table, const void *q, const int64_t *cand,
                        int32_t B, int32_t Q, int32_t K, int32_t R, int32_t k,
                        int64_t *out_ids, float *out_scores,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Re-ranking with score aggregation (Sec. 3.1: the MaxSim score is combined with the score the
 * candidate generator gave the document, through a scaling factor):
 *     total[b,j] = MaxSim(q[b], cand[b,j]) + alpha * prior[b,j]
 * ranked as in espn_rerank; out_scores holds the totals.  The factor is a plain argument (the paper's
 * is learned with the model).
 *
 *   prior  [B, K] binary32, DEVICE.   Other arguments as espn_rerank; afterwards the workspace holds
 *          all B*K totals.
 * Errors: ARG, SHAPE, UNSUPPORTED, HIP.
 */
int espn_rerank_prior(espn_table *table, const void *q, const int64_t *cand, const float *prior, float alpha,
                      int32_t B, int32_t Q, int32_t K, int32_t k,
                      int64_t *out_ids, float *out_scores,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Merge two scored lists per query (Sec. 4.3: documents re-ranked early, while the first stage was
 * still running, and documents re-ranked afterwards are combined by sorting on the score): the first
 * k entries of the union, in the order of espn_topk.  The lists need not be sorted.  A document that
 * is in both lists appears twice.
 *
 *   ids_a [B, ka] int64, scores_a [B, ka] binary32;  ids_b [B, kb], scores_b [B, kb];  all DEVICE.
 *   out_ids [B, k], out_scores [B, k], DEVICE, written.   0 <= k <= ka + kb.
 * Errors: ARG, SHAPE, HIP.
 */
int espn_merge_topk(const int64_t *ids_a, const float *scores_a, int32_t ka,
                    const int64_t *ids_b, const float *scores_b, int32_t kb,
                    int32_t B, int32_t k, int64_t *out_ids, float *out_scores, void *stream);

/*
 * Eq. 4: the largest query batch whose embedding fetch still fits the time it can hide behind,
 *     bandwidth * budget / (data size per query).
 * Host arithmetic only (no device is touched); returns 0 if bytes_per_query is not positive.
 */
double espn_batch_threshold(double bandwidth_bytes_per_s, double budget_s, double bytes_per_query);

/*
 * Wait for `stream` and report errors kernels recorded for this table since the last check:
 * returns ESPN_ERR_ID_RANGE if any candidate id was out of range, else ESPN_OK; clears the flag.
 */
int espn_table_check(espn_table *table, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Host-resident tables.  The table stays in pinned host memory (the one-GPU analogue of keeping the
 * re-ranking embeddings in a slower tier, Sec. 4); the documents a batch needs are copied to an HBM
 * staging slot ahead of scoring, on a side stream, while the previous batch is scored from the
 * other slot (Sec. 4.2: fetching overlapped with computation; Sec. 4.1: fetched straight into GPU
 * memory).  With more than two slots the slots form a ring that doubles as a cache of recently used
 * documents: a prefetch takes a document from any other slot that still holds it instead of fetching it
 * from host memory again.  Typical loop with two slots, batch n:
 *     espn_prefetch(t, cand[n+1], B, K, (n+1) % 2, side);            // returns at once
 *     espn_rerank_staged(t, n % 2, q[n], cand[n], ..., main);        // returns at once
 * Ordering between the two streams is handled inside with events: a staged re-rank waits for the
 * prefetch of its slot, and a prefetch waits for the last re-rank that read its slot and for the last
 * prefetch into every other slot.  No call here blocks the host except espn_staging_create(_ring),
 * espn_staging_counters and espn_prefetch_packed.  Calls on one table's staging slots must not be made from several host
 * threads at once.
 * ------------------------------------------------------------------------------------------- */

/*
 * Allocate the two staging slots of a table (replacing earlier ones).  Meant for host-resident
 * tables; an HBM-resident table may be staged too (the prefetch is then a stand-alone gather of the
 * batch's distinct documents, HBM to HBM).
 *   capacity_rows  embedding rows one slot can hold (each slot takes capacity_rows * dim * 2 bytes of
 *                  HBM, plus 8 bytes per document of the table for its row map).
 *   capacity_docs  distinct documents one slot can hold.
 * A prefetch that needs more raises a flag that espn_table_check reports as ESPN_ERR_NOMEM.
 * Synchronous.  Errors: ARG, NOMEM, HIP.
 */
int espn_staging_create(espn_table *table, int64_t capacity_rows, int64_t capacity_docs);

/* The same with n_slots slots, 2 <= n_slots <= 8, numbered 0 .. n_slots-1 (each of the given capacity). */
int espn_staging_create_ring(espn_table *table, int32_t n_slots, int64_t capacity_rows, int64_t capacity_docs);

/*
 * Copy every distinct document named in cand to staging slot `slot`: a document listed by several
 * queries crosses PCIe once, and a document that the last prefetch into ANOTHER slot brought in is
 * copied from there (HBM to HBM) instead of crossing PCIe again, so documents that stay popular from
 * batch to batch are fetched from the slow tier once.  Runs entirely on the GPU on `side_stream` (mark
 * distinct ids, reserve rows, copy rows).  The call waits (on the device) for the last prefetch into
 * every other slot, whatever stream that ran on.
 *   cand  [B, K] int64, DEVICE; must stay unchanged until the prefetch has run.
 * Errors: ARG, HIP, UNSUPPORTED (a table in ordinary host memory, which the device cannot read).  Ids out of
 * range are flagged as in espn_score.
 */
int espn_prefetch(espn_table *table, const int64_t *cand, int32_t B, int32_t K, int32_t slot, void *side_stream);

/*
 * The same prefetch done the other way round (the second of the two ways to bring a batch's documents
 * from the slow tier into GPU memory ahead of scoring, Sec. 4.1 / 4.2): the HOST finds the distinct
 * documents, packs their rows back to back into pinned buffers (16 threads, two buffers of 64 MiB) and
 * sends each buffer with one plain copy on `side_stream`, packing the next buffer meanwhile.  Documents that an
 * earlier call of this function left in another slot, and that slot still holds, are not packed and sent again
 * but copied from there inside HBM (the host keeps, per document, where its newest packed prefetch put it: 12
 * bytes per document of the table; a slot refilled by espn_prefetch is not trusted).  The slot ends up in the same
 * state as after espn_prefetch (espn_rerank_staged, espn_staging_counters and later espn_prefetch calls into
 * other slots work on it unchanged).
 *   cand_host  [B, K] int64, HOST; read before the call returns.
 * The table may be in pinned or in ordinary host memory (ESPN_RESIDENT_HOST_PINNED, ESPN_RESIDENT_HOST).
 * Unlike espn_prefetch this call BLOCKS the host until all but the last two buffers have been sent, and
 * its first call on a table allocates the pinned buffers and starts the packing threads (released with the
 * staging slots).  The slot's document map is written after the last row copy: if a copy cannot be enqueued
 * the call returns the error and the slot holds no document.  Its errors
 * are found on the host before anything is enqueued: ID_RANGE (an id outside the table), NOMEM (the
 * batch does not fit the slot, or no pinned memory), UNSUPPORTED (the table is HBM-resident, or a
 * document is larger than a buffer), ARG, HIP.
 */
int espn_prefetch_packed(espn_table *table, const int64_t *cand_host, int32_t B, int32_t K, int32_t slot,
                         void *side_stream);

/*
 * espn_rerank for a host-resident table: scores cand against the rows held by `slot` (which must have
 * been prefetched with the same candidates), then ranks.  Arguments as espn_rerank; afterwards the
 * workspace holds all B*K scores as binary32 [B, K].  A candidate the slot does not hold scores
 * -infinity and raises a flag (espn_table_check: ESPN_ERR_SHAPE).
 * Errors: ARG, SHAPE, UNSUPPORTED, HIP.
 */
int espn_rerank_staged(espn_table *table, int32_t slot, const void *q, const int64_t *cand,
                       int32_t B, int32_t Q, int32_t K, int32_t k,
                       int64_t *out_ids, float *out_scores,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Waits for `stream`, then reports what the last prefetch into `slot` did: out4[0] distinct documents,
 * out4[1] rows reserved, out4[2] bytes that crossed PCIe (rows not taken from another slot, times the
 * bytes of a row), out4[3] slot capacity in rows.
 * out4 is a HOST pointer to four uint64.
 */
int espn_staging_counters(espn_table *table, int32_t slot, void *stream, uint64_t *out4);

#ifdef __cplusplus
}
#endif
#endif /* ESPN_H */
