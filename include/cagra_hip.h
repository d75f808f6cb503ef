/*
 * cagra_hip.h -- C ABI of the MI355X (gfx950) CAGRA library.
 *
 * Two operations, following the paper's problem statement:
 *   build : dataset[N, dim]            -> graph[N, degree]     (Sec. III-B)
 *   search: graph, dataset, queries[B] -> ids[B, k], dists[B, k] (Sec. IV)
 * plus the exhaustive search of Eq. 1 (ground truth for recall, Eq. 2) and
 * the single build stages, exported so that each can be checked on its own.
 *
 * Conventions for every entry point
 *   - Every pointer named below is DEVICE memory owned by the caller unless it
 *     says "host".  The library never allocates or frees device memory and
 *     keeps no pointer after the call returns.  Scratch space is passed in as
 *     `workspace` (device, 256-byte aligned), sized by the matching
 *     *_workspace_bytes() function.
 *   - Matrices are row-major fp32; `ld` is the row stride in elements.  Rows
 *     are fetched with 16-byte loads (Sec. IV-B.1): base pointers must be
 *     16-byte aligned, ld a multiple of 4 and at least dim rounded up to a
 *     multiple of 4.  dim itself may be any positive number; where it is not
 *     a multiple of 4 the floats of every row (dataset and queries alike)
 *     between dim and that rounded width must be ZERO, which leaves both
 *     distances unchanged.  cagra_convert_dataset writes rows of that form.
 *   - Graphs are row-major uint32 node ids, values < N, N <= 2^31 - 1
 *     (one bit of the index word carries the parent flag, Sec. IV-B.4).
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Calls only enqueue work on that stream and return without waiting;
 *     outputs are valid once the stream has reached that point.
 *   - Return value: 0 on success, a negative cagra_status otherwise.  On any
 *     error nothing has been launched and no output has been touched.
 *   - Distances: CAGRA_L2 is the squared Euclidean distance (no root; the
 *     order of neighbours is the same), CAGRA_IP is 0 - <x, q>, so that
 *     smaller is closer for both.  Ties are ordered by smaller id.
 */
#ifndef CAGRA_HIP_H
#define CAGRA_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CAGRA_L2 = 0,
    CAGRA_IP = 1
} cagra_metric;

/* Storage type of the dataset rows given to the search (Sec. IV-C.1: lower-precision storage
 * relieves the memory-bandwidth limit).  Rows are widened to fp32 in registers and distances
 * are accumulated in fp32 whatever the storage type; queries are always fp32. */
typedef enum {
    CAGRA_F32 = 0,
    CAGRA_F16 = 1,   /* IEEE binary16 */
    CAGRA_U8 = 2     /* unsigned bytes 0..255, used as their integer values */
} cagra_dtype;

typedef enum {
    CAGRA_OK = 0,
    CAGRA_ERR_NULL_POINTER = -1,
    CAGRA_ERR_BAD_SHAPE = -2,      /* N, dim, ld, B out of range or misaligned */
    CAGRA_ERR_BAD_DEGREE = -3,     /* degree / init_degree not usable */
    CAGRA_ERR_BAD_TOPK = -4,       /* k, itopk, search_width out of range */
    CAGRA_ERR_BAD_OPTION = -5,     /* a cagra_search_opts field is not supported */
    CAGRA_ERR_WORKSPACE = -6,      /* workspace missing, misaligned or too small */
    CAGRA_ERR_HASH_CAPACITY = -7,  /* periodic-reset table cannot hold what it receives between two resets at load 7/8 */
    CAGRA_ERR_LAUNCH = -8          /* the HIP runtime refused a launch */
} cagra_status;

#define CAGRA_INVALID_ID 0xFFFFFFFFu

/* Search tunables (Sec. IV-B, IV-C).  A zero-initialised struct means "all automatic". */
typedef struct {
    uint64_t seed;            /* seed of the step-0 random sampling (Sec. IV-A step 0) */
    int32_t max_iterations;   /* I_max; 0 => 2 * ceil(itopk / search_width) + 32 */
    int32_t mode;             /* 0 automatic (Sec. IV-C.3), 1 single workgroup per query, 2 several */
    int32_t team_size;        /* lanes per distance computation: 0 automatic, else 4, 8, 16 or 32 (Sec. IV-B.1) */
    int32_t hash_bits;        /* single mode, periodic-reset table: log2 of the LDS visited table, 8..13
                                 (Sec. IV-B.3); 0 automatic (the library picks a size, not necessarily a power
                                 of two) */
    int32_t reset_interval;   /* single mode, periodic-reset table: passes between resets, 0 automatic (the
                                 largest for which both itopk + interval * search_width * degree and, for the
                                 seeds and the passes before the first reset, (interval + 1) * search_width *
                                 degree stay within 7/8 of the table) */
    int32_t wg_per_query;     /* multi mode: workgroups (workers) per query; 0 => automatic: the largest of search_width,
                                 ceil(itopk / 64) and, for batches below the number of compute units, compute units /
                                 B (at most 32); cagra_search_describe reports it */
    int32_t table_entries;    /* single mode: entries of the LDS visited table given directly (multiple of 64,
                                 256..8192); 0 => from hash_bits.  Not both. */
    int32_t dataset_type;     /* a cagra_dtype: storage type of the rows behind `dataset` (0 = fp32) */
    int32_t table_policy;     /* single mode: how the LDS visited table forgets (Sec. IV-B.3).  1: the paper's
                                 periodic reset (open addressing, cleared every reset_interval passes, top-M
                                 ids re-registered); 2: replacement (sets of four ids, a new id replaces the
                                 oldest of its set; duplicates are rejected where candidates enter the top-M
                                 list); 0: automatic = 1 if hash_bits or reset_interval is given, else 2.
                                 Results are the same for both; only the number of distances computed twice
                                 differs. */
    int32_t workgroups_per_cu; /* single mode: persistent single-wavefront workgroups per compute unit; 0 automatic,
                                 else 1..16 (clipped to what the LDS allows).  More workgroups hide more latency,
                                 fewer make each query finish sooner, which shortens the start and the end of a
                                 batch during which the device is not full. */
    int32_t waves_per_query;  /* single mode: wavefronts of one workgroup that work on one query together (the paper
                                 maps a query to a CTA of several warps, Sec. IV-C.1): 0 automatic, 1, 2 or 4.  A team
                                 shares the LDS visited table (replacement policy only) and splits the candidates of
                                 a pass; the results are those of one wavefront, bit for bit. */
    int32_t workspace_clean;  /* multi mode: 1 = the caller vouches that the workspace is clean for exactly these search
                                 arguments: cagra_search_workspace_init was run on it with them, or the last thing that
                                 touched it was a cagra_search with them (every multi-mode search hands the workspace
                                 back clean: each query has two tables, used in turn, and the workers of a search
                                 empty the one the search before filled) that has finished or precedes this call on the same stream.  The
                                 search then is one kernel launch.  0 = unknown: the search cleans the workspace first
                                 (one more launch).  A workspace that is dirty although 1 is given yields wrong results. */
    int32_t reserved;         /* 0 */
    uint32_t *stats;          /* optional device [B, 4]: passes, parents expanded, distances computed,
                                 flags (bit 0: stopped by I_max, bit 1: visited table overflowed) */
} cagra_search_opts;

/* ---- search (Sec. IV-A steps 0-3; Sec. IV-C.1 single, IV-C.2 multi) ------------------------ */

/*
 * For each of the B queries: random sampling of search_width * degree seeds,
 * then passes of {top-M update, parent selection, neighbour expansion, distance
 * of first-time candidates} until no entry of the top-M list is left
 * unexpanded or I_max passes were made; the first k of the top-M list are
 * written.  ids[B, k] / dists[B, k] come out ascending by (distance, id);
 * if fewer than k nodes were reached the tail is (CAGRA_INVALID_ID, FLT_MAX).
 * ld (in elements) must be a multiple of the elements in 16 bytes of the storage type (4 for fp32,
 * 8 for fp16, 16 for uint8) and at least dim rounded up to such a multiple; where dim is not one,
 * the elements of every DATASET row between dim and the rounded width must be zero (see
 * cagra_convert_dataset).  Queries are fp32 rows of dim elements, ld_queries >= dim, no alignment
 * or padding asked: the kernels pad their copy of the query.
 * Requirements: 1 <= k <= itopk; single mode: itopk <= 512, search_width <= 64 and
 * search_width * degree <= 2048 (beyond 256 candidates a pass takes them in chunks of 256, the
 * large-candidate-list case of Sec. IV-B.2); multi mode: see cagra_search_opts.
 * B == 0 is allowed and does nothing.
 * The workspace belongs to one call at a time: it holds the query counter (single mode) or the
 * visited tables, published lists and tickets (multi mode), so another call may use the same
 * workspace only after this call's work on its stream has finished (or behind it on the same stream).
 */
int cagra_search(const uint32_t *graph, int64_t N, int32_t degree,
                 const void *dataset /* rows of opts->dataset_type, fp32 if opts is NULL */,
                 int32_t dim, int64_t ld, cagra_metric metric,
                 const float *queries, int64_t B, int64_t ld_queries,
                 int32_t k, int32_t itopk, int32_t search_width,
                 const cagra_search_opts *opts /* host, may be NULL */,
                 uint32_t *ids_out, float *dists_out,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cagra_search_workspace_bytes(int64_t N, int32_t degree, int64_t B, int32_t k,
                                    int32_t itopk, int32_t search_width,
                                    const cagra_search_opts *opts /* host, may be NULL */);

/* Puts a workspace into the clean state a multi-mode search with these arguments expects (empty visited tables,
 * zero ticket counters, table 0 in use); a search on it may then pass opts->workspace_clean = 1 and is a single kernel launch.
 * Nothing to do, and nothing launched, when the arguments resolve to the single mode.  Same argument checks as
 * cagra_search_describe, plus the workspace checks of cagra_search. */
int cagra_search_workspace_init(int64_t N, int32_t degree, int32_t dim, int64_t B, int32_t k, int32_t itopk,
                                int32_t search_width, const cagra_search_opts *opts /* host, may be NULL */,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * cagra_search for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as cagra_search without `workspace`; the scratch memory (the query counter of the
 * single mode; visited tables, published lists and tickets of the multi mode) is a static device
 * array of CAGRA_STATIC_SCRATCH_BYTES inside the library, one per GPU, held until the process ends.
 * The call allocates and frees nothing and clears what it needs with kernels on `hip_stream`.
 * A search whose cagra_search_workspace_bytes() exceeds CAGRA_STATIC_SCRATCH_BYTES is refused with
 * CAGRA_ERR_WORKSPACE (single mode needs 256 bytes at any batch size; multi mode about
 * B * (16 * workers * degree * (max_iterations + 1) rounded up to a power of two + 512 * workers *
 * ceil(itopk_local / 64)) bytes).  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams or threads) race; issue them on one stream, or one after the other.
 */
#define CAGRA_STATIC_SCRATCH_BYTES (64u << 20)
int cagra_search_static(const uint32_t *graph, int64_t N, int32_t degree,
                        const void *dataset, int32_t dim, int64_t ld, cagra_metric metric,
                        const float *queries, int64_t B, int64_t ld_queries,
                        int32_t k, int32_t itopk, int32_t search_width,
                        const cagra_search_opts *opts /* host, may be NULL */,
                        uint32_t *ids_out, float *dists_out, void *hip_stream);

/* What a search with these arguments would run with (host function, nothing is launched):
 * the resolved mode and every automatic parameter.  Same argument checks as cagra_search. */
typedef struct {
    int32_t mode;             /* 1 single, 2 multi */
    int32_t team_size;        /* lanes per distance computation */
    int32_t table_entries;    /* visited table entries (LDS per workgroup, or device memory per query) */
    int32_t reset_interval;   /* single mode: passes between resets; 0 in multi mode (never reset) */
    int32_t max_iterations;   /* I_max */
    int32_t wg_per_query;     /* workers per query (1 in single mode) */
    int32_t itopk_local;      /* list length per worker: itopk in single mode,
                                 max(k, 32, ceil(itopk / workers)) in multi mode */
    int32_t lds_bytes;        /* dynamic LDS per workgroup */
    int32_t workgroups;       /* launch size */
    int32_t table_policy;     /* single mode: 1 periodic reset, 2 replacement; 0 in multi mode */
    int32_t waves_per_query;  /* wavefronts per workgroup (1 in multi mode) */
    int32_t reserved;
    int64_t ws_tickets_offset; /* multi mode, byte offsets into the workspace: the per-query ticket counters ([B] uint32, */
    int64_t ws_which_offset;   /* clean = 0); the words that say which of a query's two tables is in use ([B] uint32, 0 or */
    int64_t ws_tables_offset;  /* 1); the tables ([B, 2, table_entries] uint32; clean = the one in use all 0xFFFFFFFF) */
} cagra_search_plan;

int cagra_search_describe(int32_t degree, int32_t dim, int64_t B, int32_t k, int32_t itopk,
                          int32_t search_width, const cagra_search_opts *opts /* host, may be NULL */,
                          cagra_search_plan *plan_out /* host */);

/* Mode the automatic rule of Sec. IV-C.3 picks (1 single, 2 multi) for a batch of B on the
 * current device: multi when B is below the number of compute units or itopk above 512. */
int cagra_search_auto_mode(int64_t B, int32_t itopk);

/* ---- exhaustive search (Eq. 1) -------------------------------------------------------------- */

/*
 * The k nearest dataset rows of every query by computing all N distances.
 * exclude_self != 0 treats query b as dataset row (self_offset + b) and leaves
 * that row out (used for the initial k-NN graph, Sec. III-B.1).
 * ids[B, k], dists[B, k] (dists may be NULL) ascending by (distance, id).
 * Distances are accumulated one dimension after the other with fused
 * multiply-adds, so the result does not depend on tiling.  k <= 512, k <= N.
 */
int cagra_exact_search(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                       const float *queries, int64_t B, int64_t ld_queries,
                       int32_t k, int32_t exclude_self, int64_t self_offset,
                       uint32_t *ids_out, float *dists_out /* may be NULL */,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cagra_exact_search_workspace_bytes(int64_t N, int64_t B, int32_t k);

/* How the exhaustive search does its arithmetic; the result is the same bit for bit. */
typedef enum {
    CAGRA_EXACT_AUTO = 0,      /* filtered for N >= 131072 (and dim <= 8192), else plain */
    CAGRA_EXACT_PLAIN = 1,     /* every distance by the fused multiply-add chain on the vector units */
    CAGRA_EXACT_FILTERED = 2   /* approximate distances from fp16 copies on the matrix cores (MFMA) pick a few
                                  thousand candidates per query, the chain ranks those; a block of query rows for
                                  which that cannot be shown to give the exact answer (the candidate buffer
                                  overflowed, or fewer than k candidates lie below the filter threshold) is done
                                  again by the plain kernels inside the same call.  N >= 4096, dim <= 8192 */
} cagra_exact_algo;

/* cagra_exact_search with the choice of algorithm (cagra_exact_search itself is the plain one).  The
 * filtered algorithm keeps fp16 copies of dataset and queries in the workspace, hence `dim` in its size;
 * queries == dataset with equal strides is recognised and copied once.  blocks_redone_out (device, may be
 * NULL) receives the number of blocks of 2048 query rows that the plain kernels had to do again (0 with
 * the plain algorithm). */
int cagra_exact_search_ex(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                          const float *queries, int64_t B, int64_t ld_queries,
                          int32_t k, int32_t exclude_self, int64_t self_offset, cagra_exact_algo algo,
                          uint32_t *ids_out, float *dists_out /* may be NULL */,
                          uint32_t *blocks_redone_out /* device, may be NULL */,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cagra_exact_search_ex_workspace_bytes(int64_t N, int32_t dim, int64_t B, int32_t k, cagra_exact_algo algo);

/* ---- graph construction (Sec. III-B) -------------------------------------------------------- */

/*
 * dataset -> CAGRA graph of out-degree `degree`: exact k-NN graph of degree
 * init_degree (0 => 2 * degree) with rows sorted by distance (Sec. III-B.1),
 * rank-based reordering and pruning (Eq. 3), reversed graph, interleaved merge
 * (Sec. III-B.2).  degree must be even, 2 <= degree <= init_degree <= 512,
 * init_degree < N.
 */
int cagra_build(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                int32_t degree, int32_t init_degree,
                uint32_t *graph_out /* [N, degree] */,
                void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cagra_build_workspace_bytes(int64_t N, int32_t dim, int32_t degree, int32_t init_degree);

/*
 * The optimisation alone (Sec. III-B.2): sorted initial graph knn[N, init_degree]
 * -> graph_out[N, degree].  Integer work only, no dataset access.
 * The intermediate results can be read back for stage-wise checks when the
 * optional outputs are given: pruned[N, degree], reversed[N, degree] (unused
 * slots CAGRA_INVALID_ID) and reversed_len[N].
 */
int cagra_optimize(const uint32_t *knn, int64_t N, int32_t init_degree, int32_t degree,
                   uint32_t *graph_out,
                   uint32_t *pruned_out /* may be NULL */,
                   uint32_t *reversed_out /* may be NULL */,
                   uint32_t *reversed_len_out /* may be NULL */,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cagra_optimize_workspace_bytes(int64_t N, int32_t init_degree, int32_t degree);

/*
 * How the edges of a node are reordered before pruning (Sec. III-B.2).  Both count, for every
 * edge X -> Y of the initial graph, the detourable routes X -> Z -> Y of Eq. 3 and sort the list
 * by (count, initial rank); they differ in the edge weight w of Eq. 3:
 *   CAGRA_REORDER_RANK      w = position of the edge in the source's sorted initial list (what
 *                           CAGRA adopts; integer work only, no distance table);
 *   CAGRA_REORDER_DISTANCE  w = the distance (needs the distances of the initial graph's edges,
 *                           knn_dists[N, init_degree], which the exhaustive search returns).
 */
typedef enum {
    CAGRA_REORDER_RANK = 0,
    CAGRA_REORDER_DISTANCE = 1
} cagra_reorder;

/* cagra_optimize with the reordering chosen; knn_dists may be NULL for CAGRA_REORDER_RANK.
 * Same workspace as cagra_optimize. */
int cagra_optimize_ex(const uint32_t *knn, const float *knn_dists, int64_t N, int32_t init_degree,
                      int32_t degree, cagra_reorder reorder, uint32_t *graph_out,
                      uint32_t *pruned_out /* may be NULL */, uint32_t *reversed_out /* may be NULL */,
                      uint32_t *reversed_len_out /* may be NULL */,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Initial graph by NN-descent (Sec. III-B.1 names it; the details are this library's): synchronous
 * rounds in which every node pulls candidates, so the result does not depend on the order of
 * processing.  Round 0: the k best of k pseudo-random nodes (the generator of the search's step 0
 * on (seed, node, slot)).  Round t: F(x) = `sample` entries of x's list from rank
 * min(((t - 1) mod ceil(k / sample)) * sample, k - sample) on, R(x) = up to `sample` nodes y with x in
 * F(y), ordered by (rank of x in F(y), y); the new list of x is the k best of its old list and all
 * entries of the lists of F(x) and R(x), x left out.
 * knn_out[N, k], dists_out[N, k]: rows ascending by (distance, id); unused slots
 * (CAGRA_INVALID_ID, FLT_MAX).  rounds: number of rounds after round 0, < 0 automatic
 * (about log2(N) / 2 + 5); sample: 1..min(64, k), 0 automatic (32).  1 <= k <= 512, k < N.
 */
int cagra_nn_descent(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                     int32_t k, int32_t rounds, int32_t sample, uint64_t seed,
                     uint32_t *knn_out, float *dists_out,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cagra_nn_descent_workspace_bytes(int64_t N, int32_t k, int32_t sample);

/* Choices of the whole build.  A zero-initialised struct is cagra_build. */
typedef struct {
    int32_t reorder;        /* a cagra_reorder */
    int32_t initial_graph;  /* 0: exact k-NN graph (exhaustive search); 1: NN-descent */
    int32_t nnd_rounds;     /* NN-descent: rounds, 0 or < 0 automatic */
    int32_t nnd_sample;     /* NN-descent: sample, 0 automatic */
    uint64_t seed;          /* NN-descent: seed of round 0 */
    int32_t exact_algo;     /* exact initial graph: a cagra_exact_algo */
    int32_t reserved;       /* 0 */
} cagra_build_opts;

/* cagra_build with choices (opts may be NULL).  The initial graph, and for the distance-based
 * reordering its distances, live in the workspace. */
int cagra_build_ex(const float *dataset, int64_t N, int32_t dim, int64_t ld, cagra_metric metric,
                   int32_t degree, int32_t init_degree, const cagra_build_opts *opts /* host */,
                   uint32_t *graph_out /* [N, degree] */,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cagra_build_ex_workspace_bytes(int64_t N, int32_t dim, int32_t degree, int32_t init_degree,
                                      const cagra_build_opts *opts /* host */);

/* ---- reachability measures of a graph (Sec. III-A) ------------------------------------------ */

/* 2-hop node count of every node: counts_out[N] (device) = number of nodes other than X that X reaches
 * in one or two steps (at most degree + degree^2).  degree <= 64. */
int cagra_two_hop_counts(const uint32_t *graph, int64_t N, int32_t degree, uint32_t *counts_out, void *hip_stream);

/* Numbers of strongly / weakly connected components of the graph.  HOST function on a HOST copy of the
 * graph (graph_host[N, degree], ids < N): a sequential traversal, nothing is launched.  Either output may
 * be NULL.  CAGRA_ERR_WORKSPACE if host memory runs out, CAGRA_ERR_BAD_SHAPE for an id >= N. */
int cagra_count_components(const uint32_t *graph_host, int64_t N, int32_t degree,
                           int64_t *strong_out /* host */, int64_t *weak_out /* host */);

/* ---- dataset storage ------------------------------------------------------------------------- */

/* fp32 rows -> fp16 (round to nearest even), uint8 (round to nearest even, clamped to 0..255) or fp32 again
 * (a plain copy to another row stride).  src[N, dim] with stride ld_src, dst[N, dim] of dst_type with stride
 * ld_dst (both in elements).  The fp32 copy serves to pad rows: the search fetches whole rows at random and the
 * memory system fetches 64-byte sectors, so rows of 200 floats (800 bytes) cost 11 % more traffic than their bytes,
 * which a stride of 208 floats on a 64-byte aligned base avoids.  Every destination row is written in full:
 * the elements from dim up to ld_dst are set to ZERO, the form the other entry points ask of rows whose dim is
 * not a whole number of 16-byte pieces (e.g. 200 dimensions as bytes: ld_dst = 208). */
int cagra_convert_dataset(const float *src, int64_t N, int32_t dim, int64_t ld_src, cagra_dtype dst_type,
                          void *dst, int64_t ld_dst, void *hip_stream);

/* ---- misc ------------------------------------------------------------------------------------ */

/* Text for a cagra_status value (static storage, never NULL). */
const char *cagra_strerror(int code);

/* Seed of slot `slot` of query `query` as drawn by step 0 (host function; lets a caller
 * reproduce the random sampling of Sec. IV-A without running a search). */
uint32_t cagra_seed_id(uint64_t seed, uint64_t query, uint64_t slot, uint64_t N);

#ifdef __cplusplus
}
#endif
#endif /* CAGRA_HIP_H */
