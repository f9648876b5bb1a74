/*
 * gnnd.h - C ABI of the MI355X (gfx950) implementation of GPU NN-Descent (GNND)
 * and the GPU graph merge (GGM) of "Large-Scale Approximate k-NN Graph
 * Construction on GPU" (arxiv 2103.15386).
 *
 * Problem statement (Alg. 1 inputs/outputs): a reference set S of n vectors of
 * dimension d, the list length k, the sample number p and an iteration count;
 * the result is the k-NN graph G: for every object its k nearest neighbours
 * found so far, as ids with distances, ascending by (distance, id).
 *
 * Conventions for every entry point
 *  - "dev" pointers are device (HBM) pointers on the GPU that owns `stream`;
 *    "host" pointers are ordinary host memory.  The library never allocates or
 *    frees device memory: vectors, workspace and outputs belong to the caller
 *    and must outlive the context that uses them.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*).  Calls that
 *    hand scalars back to the host (statistics, the verdict on a loaded graph)
 *    synchronise the stream first; the others return after enqueueing.
 *  - Every function returns GNND_OK or a negative error code and never aborts;
 *    gnnd_last_error() gives the text.  Arguments are validated before anything
 *    is launched.
 *  - Ids are int32, 0-based row numbers of the vector array.  Distances are
 *    float32 for the float metrics and int32 for GNND_L2SQ_U8.
 *  - All random draws come from a counter-based hash of (seed, purpose, node,
 *    slot, attempt/iteration): results do not depend on thread timing, and two
 *    runs with the same seed produce the same bytes.
 */
#ifndef GNND_H_
#define GNND_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gnnd_ctx gnnd_ctx; /* opaque, host-side, owned by the library */

/* Distance (Sec. 4.2: "the specified distance metric"). */
enum {
  GNND_L2SQ_F32 = 0,    /* squared L2, float32 vectors, float32 result            */
  GNND_ANGULAR_F32 = 1, /* 1 - dot product, float32 (unit) vectors, float32 result */
  GNND_L2SQ_U8 = 2,     /* squared L2, uint8 vectors, exact int32 result           */
  GNND_CHI2_F32 = 3,    /* chi-square, sum of (a-b)^2/(a+b) over the dimensions with
                           a+b > 0, non-negative float32 vectors, float32 result   */
  GNND_COSINE_F32 = 4   /* cosine distance of float32 vectors of any length,
                           1 - a.b / sqrt(|a|^2 |b|^2), float32 result; a zero vector
                           is at distance 1 from everything (Sec. 1: the method keeps
                           NN-Descent's genericness over metrics; this one carries a
                           per-vector quantity, the squared norm, kept in 4 more bytes
                           of workspace per vector)                                  */
};

enum {
  GNND_OK = 0,
  GNND_EINVAL = -1, /* bad argument                                   */
  GNND_ENOSPC = -2, /* workspace too small                            */
  GNND_ESTATE = -3, /* call out of order (e.g. iterate before a graph) */
  GNND_EHIP = -4,   /* a HIP runtime call or kernel launch failed      */
  GNND_EIO = -5     /* a file could not be opened, read or written     */
};

/* How the cross-matching distances (Sec. 4.2) are evaluated. */
enum {
  GNND_JOIN_AUTO = 0, /* library picks                                               */
  GNND_JOIN_VALU = 1, /* per-pair float32 fused accumulation in dimension order      */
  GNND_JOIN_MFMA = 2, /* Gram-block form on the matrix cores (exact for uint8 data)  */
  GNND_JOIN_MFMA_DIRECT = 3, /* the same, every nearest-object result handed to its
                               destination list by itself (one device-wide atomic each);
                               GNND_JOIN_MFMA / AUTO collect the results per workgroup and
                               bucket of destinations first where the workspace for that is
                               affordable (n <= 2^20) and use this form beyond.  Same lists */
  GNND_JOIN_GRAM = 4  /* float32 vectors of any dimension, squared L2 / angular / cosine,
                         p <= 32: inner products on the matrix cores pick, per sample, the
                         few partners that can be its nearest one; their distances are then
                         accumulated as in GNND_JOIN_VALU.  Same results as GNND_JOIN_VALU,
                         bit for bit                                                      */
};

/* Which cross-matching results go to the list update. */
enum {
  GNND_UPDATE_SELECTIVE = 0, /* per sample only its nearest partners (Sec. 4.3, Alg. 2) */
  GNND_UPDATE_ALL_PAIRS = 1  /* every evaluated pair, both ways: the variant the paper's
                                ablation (Sec. 6.2) calls GNND-r1.  Same lists for a given
                                set of proposals, many more proposals: the proposal array
                                grows from 6p to 2p(6p - 1) slots per node, and the join
                                runs in the GNND_JOIN_VALU form only                    */
};

/* How a k-NN list is kept (Sec. 4.3, "Multiple Spinlocks"). */
enum {
  GNND_LISTS_PLAIN = 0,    /* one ascending list of k entries: the best k seen so far       */
  GNND_LISTS_SEGMENTED = 1 /* k = 32 m (k = 32, 64, 96, 128): m segments of 32 entries,
                              object v can only live in segment v % m; a list starts with
                              32 random objects of every residue class and always holds,
                              per class, the best 32 seen so far; it is handed out merged,
                              ascending by (distance, id).  For gnnd_create / gnnd_build
                              (not for merges or loaded graphs); selective update only.
                              With k = 32 the same as GNND_LISTS_PLAIN                    */
};

typedef struct gnnd_params {
  int64_t n;      /* number of vectors, k < n <= 2^27                               */
  int32_t d;      /* dimension, >= 1 (float metrics: multiple of 4 reads fastest)   */
  int32_t k;      /* list length, 2 <= k <= 128                                     */
  int32_t p;      /* sample number of Sec. 4.1, 1 <= p <= min(k, 64); the matrix-core
                     join and GNND_UPDATE_ALL_PAIRS take p <= 32                    */
  int32_t metric; /* one of the distance constants above                            */
  uint64_t seed;  /* seed of all random draws                                       */
  void* stream;   /* hipStream_t; NULL = the default stream                         */
  void* workspace_dev;    /* device scratch, 256-byte aligned, caller-owned         */
  size_t workspace_bytes; /* its size, >= gnnd_workspace_bytes()                    */
  int32_t join_path;      /* GNND_JOIN_*                                            */
  int32_t update_mode;    /* GNND_UPDATE_*; 0 = the method as published             */
  int32_t list_mode;      /* GNND_LISTS_*; 0 = plain lists                          */
  int32_t reserved;       /* 0                                                      */
} gnnd_params;

/* Counters of one iteration.  ms_* are stream times from HIP events. */
typedef struct gnnd_iter_stats {
  int32_t iter;        /* 1-based number of the iteration just finished            */
  int32_t reserved;
  uint64_t inserts;    /* list entries present now that were absent before it      */
  uint64_t dist_evals; /* distances evaluated by the cross-matching                */
  uint64_t sum_new;    /* total size of all NEW sample lists                       */
  uint64_t sum_old;    /* total size of all OLD sample lists                       */
  uint64_t proposals;  /* nearest-object results found (Alg. 2 outputs)            */
  uint64_t dropped;    /* results lost to a full proposal segment: always 0        */
  uint64_t passed;     /* results handed to the list update (after the early drop) */
  float ms_sample, ms_join, ms_update;
  float ms_handout;    /* between join and update: the pass that moves staged results into
                          the destination lists' segments (matrix-core join, n <= 2^20);
                          ~0 where results are handed on inside the join itself        */
} gnnd_iter_stats;

/* Device scratch needed for these parameters (pure host arithmetic; n, d, k, p,
 * metric are read).  Returns 0 when the parameters are invalid. */
size_t gnnd_workspace_bytes(const gnnd_params* prm);

/* Create a context over `vectors_dev`: n*d elements, row-major, float32 or
 * uint8 according to the metric, 16-byte aligned.  Validates everything, lays
 * the workspace out and clears its counters (enqueued on the stream). */
int gnnd_create(gnnd_ctx** out, const gnnd_params* prm, const void* vectors_dev);
void gnnd_destroy(gnnd_ctx* ctx);

/* Text of the last error of this context (or of the last failed gnnd_create /
 * context-free call when ctx is NULL).  Never NULL. */
const char* gnnd_last_error(const gnnd_ctx* ctx);

/* Which evaluation of the cross-matching distances (Sec. 4.2) this context
 * uses: GNND_JOIN_VALU, GNND_JOIN_MFMA or GNND_JOIN_GRAM (GNND_JOIN_AUTO resolved
 * at creation: the int8 matrix-core form is taken when it is exact - squared
 * L2, d <= 128, p <= 32, uint8 vectors or float32 vectors holding only integers
 * 0..255; other float32 vectors take GNND_JOIN_GRAM where it applies (squared
 * L2, angular, cosine; p <= 32; selective update); GNND_JOIN_VALU otherwise).
 * Negative on a NULL context. */
int gnnd_join_path(const gnnd_ctx* ctx);

/* Stage timing without synchronising inside the loop.  gnnd_set_profiling(ctx,
 * iterations) opens a recording window of that many iterations (at least 64;
 * at most 65536; 0 switches profiling off); the HIP events of the window are
 * created by this call.  While profiling is on, every iteration that is run
 * without statistics (gnnd_iterate with NULL, gnnd_build) records four events on
 * the stream - before sampling, before the cross-matching, behind the
 * cross-matching kernel (in front of the pass that moves staged results into
 * the destinations' segments, where there is one), before the update, after it.  An iteration that finds the window full runs as usual, is not
 * recorded and is counted as missed.
 * gnnd_get_stage_ms synchronises the stream, returns the number of recorded
 * iterations, the number of missed ones and the summed milliseconds of each
 * stage over the recorded ones (all host pointers, required), and starts a new
 * window of the same size. */
int gnnd_set_profiling(gnnd_ctx* ctx, int iterations);
int gnnd_get_stage_ms(gnnd_ctx* ctx, int32_t* count_host, int32_t* missed_host,
                      float* ms_sample_host, float* ms_join_host, float* ms_handout_host,
                      float* ms_update_host);

/* Alg. 1, first loop: every list gets k distinct random objects other than the
 * node itself, with their distances, ascending by (distance, id), all flagged
 * NEW.  Resets the iteration counter to 0. */
int gnnd_init_random(gnnd_ctx* ctx);

/* One pass of the Alg. 1 loop body: ParallelSample (Sec. 4.1), cross-matching
 * (Sec. 4.2), selective update and list insertion (Sec. 4.3).  `stats_host`
 * may be NULL (then nothing is copied back and the call does not synchronise). */
int gnnd_iterate(gnnd_ctx* ctx, gnnd_iter_stats* stats_host);

/* The three stages of gnnd_iterate one at a time, in this order, for step-wise
 * checks: sampling; cross-matching + nearest-object selection; list update
 * (which ends the iteration and may return its statistics). */
int gnnd_step_sample(gnnd_ctx* ctx);
int gnnd_step_join(gnnd_ctx* ctx);
int gnnd_step_update(gnnd_ctx* ctx, gnnd_iter_stats* stats_host);

/* Alg. 1 as a whole: gnnd_init_random, then up to max_iters iterations.
 * delta > 0 additionally stops after an iteration with fewer than
 * delta * n * k inserts (not in the paper; 0 = fixed iteration count).
 * `last_host` (may be NULL) receives the statistics of the last iteration run. */
int gnnd_build(gnnd_ctx* ctx, int32_t max_iters, float delta, gnnd_iter_stats* last_host);

/* Copy the graph out: n*k ids, n*k distances (float32 or int32 by metric) and
 * n*k NEW flags (0/1), row per node, ascending by (distance, id).  Any of the
 * three device pointers may be NULL. */
int gnnd_get_graph(gnnd_ctx* ctx, int32_t* ids_dev, void* dist_dev, uint8_t* isnew_dev);

/* Load a graph (same layout; rows must be sorted by (distance, id) and hold k
 * distinct ids) and set the iteration counter: continuing from a saved graph
 * gives the same bytes as an uninterrupted run.  Ids are checked on the device:
 * one outside 0..n-1, or a node in its own list, gives GNND_EINVAL and leaves
 * the context without a graph.  Synchronises the stream. */
int gnnd_set_graph(gnnd_ctx* ctx, const int32_t* ids_dev, const void* dist_dev,
                   const uint8_t* isnew_dev, int32_t iter);

/* Sample lists of the last gnnd_step_sample / gnnd_iterate (Sec. 4.1): n rows of
 * 2p ids ascending, unused tail -1, and the n list sizes, per kind. */
int gnnd_get_samples(gnnd_ctx* ctx, int32_t* new_dev, int32_t* cnt_new_dev, int32_t* old_dev,
                     int32_t* cnt_old_dev);

/* Nearest-object results of the last gnnd_step_join (Alg. 2 outputs) that can
 * still enter a list, i.e. whose distance does not exceed the distance of the
 * destination list's last entry: three arrays of n*6p slots.  Results are
 * grouped by destination list in no particular order; u_dev = list to insert
 * into, or -1 for an unused slot; v_dev = object to insert; dist_dev = its
 * distance (float32 / int32 by metric).  Valid between join and update only. */
int gnnd_get_proposals(gnnd_ctx* ctx, int32_t* u_dev, int32_t* v_dev, void* dist_dev);

/* GGM (Sec. 5.1, Alg. 3): merge the k-NN graph G1 of S1 (n1 vectors at
 * vec1_dev) and G2 of S2 (n2 vectors at vec2_dev) into the graph of S1 u S2,
 * prm->n = n1 + n2, output rows 0..n1-1 = S1 then S2.
 * Ids are ids of a collection of id_space objects in which S1 is the range
 * [base1, base1 + n1) and S2 is [base2, base2 + n2) (disjoint; for two halves
 * of one array: base1 = 0, base2 = n1, id_space = n).  Input lists may also
 * hold ids outside both ranges (left by an earlier merge with a third shard,
 * Sec. 5.1): such entries are frozen - they compete for their place with their
 * stored distance but are never sampled.  A list must not yet hold ids of the
 * other set.  Needs n + id_space <= 2^30.
 * Each list keeps its first ceil(k/2) entries, the rest is set aside and
 * replaced by floor(k/2) random objects of the other set flagged NEW; `iters`
 * GNND iterations then evaluate only pairs from different sets (and no
 * NEW x NEW pairs); finally each list is the best k of the refined list and its
 * set-aside half, in collection ids, ascending by (distance, id).
 * Synchronises when stats_host (array of `iters` entries, may be NULL) is given. */
int gnnd_merge(const gnnd_params* prm, const void* vec1_dev, int64_t n1, int64_t base1,
               const void* vec2_dev, int64_t n2, int64_t base2, int64_t id_space,
               const int32_t* ids1_dev, const void* dist1_dev, const int32_t* ids2_dev,
               const void* dist2_dev, int32_t iters, int32_t* ids_out_dev, void* dist_out_dev,
               gnnd_iter_stats* stats_host);

/* Incremental construction (Sec. 5.1, its remark on data that arrive later): a
 * batch S2 of n2 new vectors (vec2_dev) joins the collection S1 of n1 vectors
 * (vec1_dev) whose graph G1 (ids1_dev, dist1_dev: n1*k, ids 0..n1-1) exists.
 * GNND first builds the sub-graph of S2 on its own (random initial graph and
 * build_iters iterations, with seed + 1), then GGM joins it into G1
 * (gnnd_merge with base1 = 0, base2 = n1, id_space = n, merge_iters iterations,
 * with seed).  prm->n = n1 + n2; the workspace for prm serves both steps.
 * Output as gnnd_merge: n*k entries, rows 0..n1-1 = S1 then S2, ids 0..n-1
 * with the new objects numbered n1..n-1.  Both sets need more than k objects.
 * Enqueues on prm->stream and returns without synchronising. */
int gnnd_append(const gnnd_params* prm, const void* vec1_dev, int64_t n1, const int32_t* ids1_dev,
                const void* dist1_dev, const void* vec2_dev, int64_t n2, int32_t build_iters,
                int32_t merge_iters, int32_t* ids_out_dev, void* dist_out_dev);

/* Out-of-core construction (Sec. 5.1) on one GPU.  The collection of prm->n
 * vectors stays in pinned host memory (vectors_host, n*d elements); it is cut
 * into `shards` shards of floor(n/shards) consecutive rows (the last takes the
 * remainder).  Every shard is built on its own (gnnd_build with seed + shard
 * number, build_iters iterations), then every pair of shards is merged once by
 * GGM (merge number m, in rounds of disjoint pairs, with seed + 1000 + m and
 * merge_iters iterations) and stored back as the two shards' sub-graphs.  Only
 * two shards are resident at a time; prm->workspace_dev / workspace_bytes is a
 * device arena of gnnd_sharded_arena_bytes() bytes holding two alternating
 * slots plus the scratch of one merge; uploads and downloads run on copy_stream
 * (a second stream, required) while prm->stream computes.
 * ids_host / dist_host (pinned host memory, n*k each) receive the final graph
 * in collection ids and hold the sub-graphs in between.  The call returns after
 * both streams have drained.  stats_host may be NULL. */
typedef struct gnnd_shard_stats {
  int32_t builds, merges;
  float ms_build; /* compute-stream time of the shard builds (events)  */
  float ms_merge; /* compute-stream time of all pairwise merges        */
  float ms_total; /* host wall time of the whole call, copies included */
  float reserved;
} gnnd_shard_stats;
size_t gnnd_sharded_arena_bytes(const gnnd_params* prm, int32_t shards);
int gnnd_build_sharded(const gnnd_params* prm, const void* vectors_host, int32_t shards,
                       int32_t build_iters, int32_t merge_iters, int32_t* ids_host,
                       void* dist_host, void* copy_stream, gnnd_shard_stats* stats_host);

/* The same out-of-core construction with the collection and the graph in files
 * (Sec. 5.1: sub-graphs are saved to external storage, and reading and writing
 * them runs beside the GPU's work).  vectors_path: n*d elements, row-major, read
 * only.  ids_path / dist_path: created or overwritten, n*k int32 and n*k
 * distances; they hold the sub-graphs in between and the final graph (collection
 * ids) at the end.  staging_host: pinned host memory of staging_bytes (>= 1 MiB;
 * a few hundred MiB keeps the pieces large), the only host buffer used: every
 * transfer is cut into pieces of half that size; host functions on a stream the
 * call creates for itself read or write one half while copy_stream moves the
 * other half over the bus and prm->stream computes.  Procedure, seeds, arena and
 * result are those of gnnd_build_sharded: the files end up holding the same
 * bytes as its ids_host / dist_host.  Files are checked and sized before any
 * GPU work; a later read or write failure returns GNND_EIO once all streams
 * have drained (the files' contents are then undefined). */
int gnnd_build_sharded_files(const gnnd_params* prm, const char* vectors_path, int32_t shards,
                             int32_t build_iters, int32_t merge_iters, const char* ids_path,
                             const char* dist_path, void* staging_host, size_t staging_bytes,
                             void* copy_stream, gnnd_shard_stats* stats_host);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): gnnd_build + gnnd_get_graph
 * in one call whose scratch is a static device array inside the library instead
 * of a caller's workspace.  prm->workspace_dev / workspace_bytes are ignored;
 * vectors_dev (n*d, as for gnnd_create) and the outputs ids_out_dev (n*k int32)
 * and dist_out_dev (n*k float32 / int32 by metric) are the caller's.  Random
 * initial graph, then exactly max_iters iterations; same result as gnnd_create +
 * gnnd_build + gnnd_get_graph with the same parameters.
 *  - The array holds GNND_STATIC_SCRATCH_BYTES = 64 MiB per GPU (about 12,000
 *    nodes at k = p = 32, d = 128); parameters whose gnnd_workspace_bytes() need
 *    exceeds it are refused with GNND_ENOSPC before anything is launched.
 *  - Nothing is allocated or freed, on the device or on the host, and the call
 *    never synchronises: it enqueues on prm->stream and returns.  The device
 *    that owns the stream must be the current device.  The first call on a
 *    device looks the array's address up (the HIP runtime sets the array up on
 *    that device at this point, and the device holds it until the process
 *    ends): make one call per device before capturing or entering a loop that
 *    must not touch the allocator.
 *  - GNND_JOIN_AUTO takes the int8 matrix-core join for uint8 vectors (d <= 128)
 *    and never for float32 vectors (deciding that float data are byte valued
 *    would need a synchronisation: they take GNND_JOIN_GRAM or GNND_JOIN_VALU);
 *    GNND_JOIN_MFMA with float32 vectors is refused.
 *  - All calls on one GPU share that GPU's array: two calls that overlap in time
 *    on one GPU (different streams or threads) race.  Each call clears what it
 *    needs cleared; nothing is kept from one call to the next. */
#define GNND_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int gnnd_build_static(const gnnd_params* prm, const void* vectors_dev, int32_t max_iters,
                      int32_t* ids_out_dev, void* dist_out_dev);

/* Exact K nearest neighbours by exhaustive search (the ground truth of
 * Recall@K, Sec. 6.1) of nq query nodes (ids in queries_dev) against all n
 * vectors, the node itself excluded: nq*K ids and distances ascending by
 * (distance, id).  K <= 64.  Needs no context and no workspace.  A query id
 * outside 0..n-1 (and any rank beyond n-1 neighbours) gets id -1 and the
 * largest distance. */
int gnnd_exact_knn(const void* vectors_dev, int64_t n, int32_t d, int32_t metric,
                   const int32_t* queries_dev, int64_t nq, int32_t K, int32_t* ids_out_dev,
                   void* dist_out_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GNND_H_ */
