/*
 * ann.h -- C ABI of the MI355X (gfx950) graph-ANNS library.
 *
 * The library builds a Vamana/DiskANN-style proximity graph by deterministic
 * prefix-doubling batch insertion (Alg. 3 of the paper: batchBuild /
 * BatchInsert) and answers batched k-NN queries with greedy beam search
 * (Alg. 1); with the same kernels it builds and searches the layered index of
 * Sec. 4.2 and builds the clustering-based graph of Sec. 4.3 (both further
 * down).  Every step runs in hand-written HIP kernels on one GPU.
 *
 * Conventions shared by all calls
 *   - "dev" pointers are HIP device pointers, "host" pointers are ordinary
 *     host memory.  Matrices are row-major and contiguous.  Device base
 *     pointers must be 16-byte aligned.
 *   - Distances: squared Euclidean (ANN_L2SQ, any dtype) or negative inner
 *     product (ANN_MIPS, ANN_F32 only).  Smaller is closer (Sec. 2).  For
 *     u8/i8 the distance is the exact int32; for f32 it is computed in fp32.
 *   - Every "closest" is decided under the total order (distance, id).
 *   - A graph is n rows of R uint32 ids (fixed-length edge lists, Sec. 4.5);
 *     valid neighbours come first, unused slots hold ANN_NONE.
 *   - Vertex ids are < 2^31.  Supported row sizes: u8/i8 1 <= d <= 512;
 *     f32 needs d % 4 == 0 and d <= 256.  u8/i8 rows whose size is not a
 *     multiple of 16 bytes are copied once, per points array, into zero-
 *     padded rows that the graph object keeps (n x stride bytes of device
 *     memory, stride = d rounded up to 16, or to a power of two where that
 *     costs at most a quarter more); queries are copied per call.  The
 *     points array must not change while a graph built on it is in use.
 *   - Every function returns ANN_OK (0) or a negative ann_status; on error
 *     outputs are untouched, *out handles are NULL and ann_last_error()
 *     describes the failure.  No exception or abort crosses this boundary.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).
 *   - The library allocates its own scratch and frees it before returning,
 *     except for what an object keeps until it is freed: the adjacency rows,
 *     the padded copies named above, and the scratch of ann_insert_batch /
 *     ann_insert_points (sized for the largest batch so far).  The memory
 *     comes from hipMalloc / hipFree, or from the `alloc` / `free` callbacks
 *     of ann_build_opts / ann_hnsw_opts, which the object then keeps for all
 *     its later allocations and for its own release (the clustering-based
 *     builder always uses hipMalloc).  The caller owns every buffer it
 *     passes in.
 *   - Calls that use one graph or index object must be issued on one stream
 *     (or be ordered by the caller): the object's padded query copy and
 *     insertion scratch are shared by all calls on it.
 *   - With ANN_TRACE_BUILD set in the environment, ann_build,
 *     ann_insert_points and ann_hcnng_build print a wall-clock breakdown of
 *     their phases on stderr (the clustering-based builder waits for the
 *     stream between phases to do so: for measurement only).
 */
#ifndef ANN_H
#define ANN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ANN_NONE 0xFFFFFFFFu

typedef enum { ANN_U8 = 0, ANN_I8 = 1, ANN_F32 = 2 } ann_dtype;
typedef enum { ANN_L2SQ = 0, ANN_MIPS = 1 } ann_metric;

typedef enum {
  ANN_OK = 0,
  ANN_EINVAL = -1, /* null pointer, zero size, k > L, unsupported shape ... */
  ANN_ENOMEM = -2, /* a device or host allocation failed                    */
  ANN_EHIP = -3,   /* a HIP call failed; text in ann_last_error()           */
  ANN_EINTERNAL = -4
} ann_status;

/* Opaque graph handle.  Owns the device memory of the n x R adjacency rows. */
typedef struct ann_graph ann_graph;

/* Device-memory callbacks (Sec. 2's problem statement leaves memory to the
 * caller; a host program that runs its own caching allocator hands it in
 * here).  `alloc` returns a device pointer aligned to at least 256 bytes that
 * is valid on `stream` (the stream of the call that allocates), or NULL when
 * it has no memory: the call then fails with ANN_ENOMEM.  `free` takes back a
 * pointer `alloc` returned; the library has waited for its own work on that
 * memory, except in ann_graph_free / ann_hnsw_free, which do not wait for
 * searches the caller still has in flight.  Neither may call into this
 * library.  Both are called on the thread of the API call that needs them. */
typedef void* (*ann_alloc_fn)(size_t bytes, void* stream, void* user);
typedef void (*ann_free_fn)(void* ptr, void* user);

/* Optional knobs of ann_build.  Zero-initialise, then set what is needed.   */
typedef struct {
  uint64_t batch_cap;    /* theta, the batch-size bound of Sec. 3.1; 0 = max(1, n/50)  */
  uint32_t start;        /* start vertex s, used only when use_start is non-zero       */
  uint32_t use_start;    /* zero: s = point nearest the mean (ann_start_vertex)        */
  const uint32_t* order; /* host, n-1 ids: insertion order; NULL = seeded shuffle      */
  uint32_t visited_cap;  /* slots per search for the visited list; 0 = max(256, 4L).
                            A search that visits more moves its list to a spill chunk;
                            if that fails too the search is redone with enough room, so
                            the result never depends on this value.                    */
  uint64_t spill_cap;    /* keys of spill space for such lists; 0 = default            */
  uint32_t hash_bits;    /* log2 size of the per-search visited filter in LDS; 0 = auto.
                            The filter only saves work; results do not depend on it.   */
  uint64_t max_rounds;   /* stop after this many batches (0 = all): partial builds     */
  uint32_t collect_stats;/* non-zero: count hops, distance evaluations, ... (slower)   */
  ann_alloc_fn alloc;    /* device memory for the graph and all scratch; NULL = hipMalloc */
  ann_free_fn free;      /* its counterpart; both or neither                           */
  void* alloc_user;      /* passed to both                                             */
  uint32_t step1_parts;  /* 0: batches of 8,192 points and more run step 1 of BatchInsert in
                            three parts side by side (see ann_stats); 1: always in one part.
                            The graph does not depend on it.                            */
} ann_build_opts;

typedef struct {
  uint64_t n;
  uint32_t d;
  uint32_t R;
  uint32_t dtype;
  uint32_t metric;
  uint32_t start;
  uint64_t rounds; /* batches inserted so far */
} ann_graph_info_t;

typedef struct {
  uint64_t searches;    /* greedy searches run                                   */
  uint64_t hops;        /* vertices processed, summed over searches (|V|)        */
  uint64_t evals;       /* distances taken in searches, re-evaluations included  */
  uint64_t prunes;      /* step-1 prunes                                         */
  uint64_t reprunes;    /* step-2 prunes of overflowing rows                     */
  uint64_t appends;     /* step-2 rows that only appended                        */
  uint64_t edges;       /* reverse edges grouped                                 */
  uint64_t prune_evals; /* pair distances taken inside prune                     */
  uint64_t redone;      /* searches redone because the visited list fit nowhere  */
  uint64_t restarts;    /* builds started over in synchronised mode for that     */
  uint64_t rounds;
  uint64_t passes;      /* searches: 8-vertex distance passes                    */
  uint64_t survivors;   /* searches: candidates inserted into a beam             */
  uint64_t insert_hops; /* searches: hops that inserted at least one candidate   */
  /* device time per phase.  A batch of 8,192 points or more runs step 1 in three parts side by
   * side (a part that is through its searches prunes while the others still search):
   * ms_search lasts from a batch's start until the last of its searches is over, ms_prune from
   * then until its last prune is over.                                                      */
  double ms_search, ms_prune, ms_sort, ms_merge, ms_total;
  uint64_t search_launches;  /* launches of the search kernel in batches (with statistics on) */
  double ms_search_launches; /* their durations added up; launches of one batch overlap      */
} ann_stats;

/*
 * batchBuild(P, s, R, L) of Alg. 3.  Inserts the points in a seeded random
 * order in batches of size 2, 4, 8, ... bounded by theta.  Per batch:
 * every point runs greedySearch (Alg. 1) with beam width L from s over the
 * graph as it stood before the batch; its visited set is pruned to at most R
 * out-neighbours with the alpha rule of Sec. 4.1 (drop p' when
 * alpha*d(p*,p') <= d(p,p')); the new edges are reversed, grouped by
 * destination with an on-device radix sort, appended in batch order, and rows
 * that exceed R are pruned again.
 *
 *   points_dev  n x d elements of `dtype` (device)
 *   alpha       > 0 (must be <= 1 for ANN_MIPS, Appendix A).  For u8/i8 it is
 *               quantised to llround(alpha * 65536) / 65536, which must be
 *               at least 1 / 65536.
 *   seed        drives the insertion order: the ids other than s in ascending
 *               order, shuffled by Fisher-Yates from the front (step i exchanges
 *               positions i and i + mulhi64(r, m - i), r the next SplitMix64(seed)
 *               output), so the build starts while the order is still drawn
 *   opts        may be NULL
 *   *out        receives the graph; free with ann_graph_free
 * Blocks until the build is complete.
 */
int ann_build(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
              uint32_t R, uint32_t L, float alpha, uint64_t seed, const ann_build_opts* opts,
              void* stream, ann_graph** out);

/*
 * BatchInsert(P') of Alg. 3 on an existing graph: inserts the `b` points whose
 * ids are in ids_host (all < n, none twice, none equal to the start vertex,
 * none with out-neighbours already: ANN_EINVAL otherwise) as ONE batch.  `points_dev` must be the array the graph was built
 * over.  Blocks until done.
 */
int ann_insert_batch(ann_graph* g, const void* points_dev, const uint32_t* ids_host, uint64_t b,
                     uint32_t L, float alpha, void* stream);

/*
 * Streaming insertion: the graph, which holds the points 0..n-1, takes in the
 * points n..n_total-1 with BatchInsert of Alg. 3, in batches that carry on the
 * prefix-doubling schedule of ann_build (Sec. 3.1): min(present + 2, theta,
 * left) points at a time, `present` counting the graph's points other than
 * the start vertex.  The start vertex stays what it is.  Deterministic like
 * the build: the result depends on the arguments only.
 *   points_dev  n_total x d elements of the graph's dtype (device); its first
 *               n rows are the points the graph holds (the same array as
 *               before, or a copy that was extended)
 *   n_total     >= the graph's n and < 2^31; equal: nothing happens
 *   seed        drives the order of the new ids (the shuffle of ann_build
 *               applied to the list n, n+1, ..., n_total-1)
 *   opts        may be NULL.  Read: batch_cap (theta; 0 = max(1, n_total/50)),
 *               order (n_total - n ids, every new id once, host), max_rounds.
 *               The other fields keep the values given to ann_build.
 * The adjacency rows move to a larger allocation when the capacity is
 * exceeded (see ann_graph_reserve): pointers from ann_graph_device_rows are
 * stale after the call, and no other call on this graph may be in flight.
 * After an error the graph may hold some of the new points, inserted or as
 * unreachable vertices with empty rows.  Blocks until done.
 */
int ann_insert_points(ann_graph* g, const void* points_dev, uint64_t n_total, uint32_t L, float alpha,
                      uint64_t seed, const ann_build_opts* opts, void* stream);

/*
 * Room for n_cap points in the graph's arrays, so that ann_insert_points up
 * to that size moves nothing.  (Without it the capacity grows by half each
 * time it is exceeded.)  Never shrinks.  Blocks; invalidates the pointer of
 * ann_graph_device_rows when it grows.
 */
int ann_graph_reserve(ann_graph* g, uint64_t n_cap, void* stream);

/*
 * greedySearch(q, s, L, k) of Alg. 1 for nq queries (one wavefront each).
 *   queries_dev  nq x d elements of the graph's dtype (device)
 *   ids_dev      nq x k uint32 (device): the k closest found, ascending by
 *                (distance, id); ANN_NONE where fewer than k were reached
 *   dists_dev    nq x k int32 (u8/i8) or float (f32); INT32_MAX / +inf padding
 * Requires 1 <= k <= L <= 2048 (the beam of Sec. 4.5's sweeps; builds take L <= 512).
 * Asynchronous on `stream`.
 */
int ann_search(const ann_graph* g, const void* points_dev, const void* queries_dev, uint64_t nq,
               uint32_t k, uint32_t L, uint32_t* ids_dev, void* dists_dev, void* stream);

/*
 * The same search with the (1 + eps) pruning of Sec. 4.5: a vertex is searched only while its
 * distance to the query is within a factor 1 + eps of the current k-th nearest candidate.
 * The test is made before the closest unprocessed beam member is expanded, once the beam
 * holds k entries, and its first failure ends the search (the beam is sorted and its k-th
 * distance never grows).  Distances are the ones the library computes (squared for ANN_L2SQ);
 * u8/i8: d * 2^16 > d_k * (2^16 + round(eps * 2^16)) in 64-bit integers; f32: d > d_k + eps * |d_k|
 * in fp32 (which also covers the negative values of ANN_MIPS).  Equality passes.
 *   eps   0 <= eps < 16384 (the paper never uses more than 0.25); a negative eps switches the
 *         rule off and makes the call identical to ann_search
 * Other arguments, outputs and errors as ann_search.  Asynchronous on `stream`.
 */
int ann_search_eps(const ann_graph* g, const void* points_dev, const void* queries_dev, uint64_t nq,
                   uint32_t k, uint32_t L, float eps, uint32_t* ids_dev, void* dists_dev, void* stream);

/*
 * ann_search_eps for callers that cannot allocate device memory: code under HIP graph capture,
 * serving loops, harnesses that forbid hipMalloc.  It calls no allocator of any kind.  The one
 * buffer the search needs beyond its inputs and outputs, the zero-padded copy of the queries
 * for u8/i8 rows whose size is not a multiple of 16 bytes, is a device array inside the library
 * of ANN_NOALLOC_SCRATCH_MIB MiB, which every GPU the library runs on holds until the process
 * ends.  (Rows that need no padding use no scratch at all.)
 *   - nq * padded row size must fit the array: ANN_EINVAL otherwise, with the largest nq in the
 *     message (65,536 queries for rows padded to 128 bytes).
 *   - For padded rows the graph must already hold the padded copy of `points_dev`: ann_build
 *     makes it, and so does one call of ann_search; ANN_EINVAL otherwise.
 *   - All calls on one GPU share the array: calls that overlap in time on one GPU (two streams,
 *     two threads, two graphs) race on it.  The caller orders them.
 * Arguments, results and errors otherwise as ann_search_eps (eps < 0: plain ann_search).
 * Asynchronous on `stream`.
 */
#define ANN_NOALLOC_SCRATCH_MIB 8
int ann_search_noalloc(const ann_graph* g, const void* points_dev, const void* queries_dev, uint64_t nq,
                       uint32_t k, uint32_t L, float eps, uint32_t* ids_dev, void* dists_dev, void* stream);

/* Start vertex used by ann_build when none is given: the point nearest
 * (squared L2) to the mean of all points, smallest id on ties.  Exact for
 * u8/i8; fp64 for f32.  Blocks.                                             */
int ann_start_vertex(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, void* stream,
                     uint32_t* start_out);

/* Wrap adjacency rows given on the host (n x R, ANN_NONE padded) as a graph. */
int ann_graph_from_host(const uint32_t* rows_host, uint64_t n, uint32_t d, ann_dtype dtype,
                        ann_metric metric, uint32_t R, uint32_t start, ann_graph** out);

/* Copy the n x R adjacency rows to host memory.  Blocks.                    */
int ann_graph_copy_neighbors(const ann_graph* g, uint32_t* rows_host);

/* Device pointer to the n x R adjacency rows (owned by the graph).          */
const uint32_t* ann_graph_device_rows(const ann_graph* g);

int ann_graph_info(const ann_graph* g, ann_graph_info_t* info);
int ann_get_stats(const ann_graph* g, ann_stats* stats); /* cumulative over build + inserts */
/* Switches the counters of ann_get_stats on or off for the calls that follow
 * (builds start with opts->collect_stats).  With them on, searches on this
 * graph add their hops and distance evaluations too.                        */
int ann_graph_set_stats(ann_graph* g, int on);
/* Size of the visited filter of the searches that follow on this graph, as
 * opts->hash_bits of ann_build (log2 of the size in 32-bit words, 4..13; 0 =
 * chosen from the beam width).  For the sizing study of Sec. 4.5: results never
 * depend on it, only the number of repeated distance evaluations does.       */
int ann_graph_set_filter_bits(ann_graph* g, uint32_t hash_bits);
void ann_graph_free(ann_graph* g);

/* Stable LSD radix sort of `count` 64-bit keys by bits [32, 32+key_bits) only
 * (the grouping step of BatchInsert; exposed for tests).  In place on
 * keys_dev; blocks.                                                         */
int ann_sort_edges(uint64_t* keys_dev, uint64_t count, uint32_t key_bits, void* stream);

/* ------------------------------------------------------------------------
 * Layered index (Sec. 4.2, ParlayHNSW): layer l holds the points whose level
 * is at least l; every layer is built with the batch insertion of Alg. 3
 * (one batch insertion per layer); the degree bound is m above the bottom
 * layer and 2m on it (appendix, parameter paragraph); prune is the alpha rule
 * of Sec. 4.1 on every layer.
 *   level of point i   with r = the (i+1)-th output of SplitMix64(seed): the
 *                      largest l with r <= floor((2^64 - 1) / m^l)
 *   entry point        the point of the highest level, smallest id on ties;
 *                      present on every layer from the start, never inserted
 *   order, batches     as ann_build, the entry point in the start vertex's
 *                      place
 *   one batch          every point walks down from the entry point: on a
 *                      layer above its level a search with beam 1 over the
 *                      layer as it stood before the batch; on its own layers
 *                      BatchInsert with beam efc; either way the closest
 *                      vertex found is where it enters the layer below
 * ------------------------------------------------------------------------ */
typedef struct ann_hnsw ann_hnsw;

typedef struct {
  uint64_t batch_cap;     /* theta; 0 = max(1, n/50)                              */
  const uint32_t* order;  /* host, n-1 ids (all but the entry point); NULL = seeded */
  const uint32_t* level;  /* host, n levels (each <= 63); NULL = drawn from seed   */
  uint64_t max_rounds;    /* stop after this many batches (0 = all)                */
  uint32_t collect_stats; /* non-zero: counters and phase times (slower)           */
  ann_alloc_fn alloc;     /* device memory for the index and all scratch; NULL =    */
  ann_free_fn free;       /* hipMalloc / hipFree; both or neither                   */
  void* alloc_user;
} ann_hnsw_opts;

typedef struct {
  uint64_t n;
  uint32_t d;
  uint32_t m;
  uint32_t dtype;
  uint32_t metric;
  uint32_t top;   /* highest layer */
  uint32_t entry; /* entry point   */
  uint64_t rounds;
} ann_hnsw_info_t;

/* Builds the index over points_dev (n x d, device; same types and sizes as
 * ann_build, with R = 2m, i.e. 2 <= m <= 256).  efc is the beam width of the
 * insertions.  The upper layers keep copies of their points (a fraction
 * 1/(m-1) of the input).  Blocks until done.                                 */
int ann_hnsw_build(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                   uint32_t m, uint32_t efc, float alpha, uint64_t seed, const ann_hnsw_opts* opts,
                   void* stream, ann_hnsw** out);

/* Streaming insertion into the layered index: it takes in the points
 * n..n_total-1 the way ann_insert_points does for the flat graph (the build's
 * schedule carried on, BatchInsert per layer).  A new point's level follows
 * the index's rule (the seed given to ann_hnsw_build; 0 for an index from
 * ann_hnsw_from_host) but is at most the index's highest layer, whose entry
 * point stays.  opts: batch_cap, order (n_total - n new ids), level (n_total -
 * n levels, in place of the rule), max_rounds.  seed drives the order.  Every
 * batch waits on the host once; blocks until done.                           */
int ann_hnsw_insert_points(ann_hnsw* h, const void* points_dev, uint64_t n_total, uint32_t efc, float alpha,
                           uint64_t seed, const ann_hnsw_opts* opts, void* stream);

/* Wraps an index given on the host: level_host (n), the entry point (a point
 * of the highest level), and rows_host[l] for l = 0..max level, each n x
 * (l ? m : 2m) adjacency rows of point ids, ANN_NONE padded (the rows of
 * points below layer l are ignored).  points_dev as ann_hnsw_build.  Blocks. */
int ann_hnsw_from_host(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                       uint32_t m, const uint32_t* level_host, uint32_t entry,
                       const uint32_t* const* rows_host, void* stream, ann_hnsw** out);

/* Queries: beam 1 from the entry point down to layer 1, then greedySearch of
 * Alg. 1 on layer 0 from the vertex reached (with the (1 + eps) rule of
 * ann_search_eps when eps >= 0).  Arguments and outputs as ann_search_eps;
 * points_dev is the array the index was built over.  Asynchronous on stream. */
int ann_hnsw_search(const ann_hnsw* h, const void* points_dev, const void* queries_dev, uint64_t nq,
                    uint32_t k, uint32_t L, float eps, uint32_t* ids_dev, void* dists_dev, void* stream);

int ann_hnsw_info(const ann_hnsw* h, ann_hnsw_info_t* info);
/* n levels to host memory.                                                   */
int ann_hnsw_copy_levels(const ann_hnsw* h, uint32_t* level_host);
/* Number of points on a layer (n for layer 0).                               */
int ann_hnsw_layer_size(const ann_hnsw* h, uint32_t layer, uint64_t* count);
/* A layer to host memory: ids_host receives the ids of its count points in
 * ascending order, rows_host their count x (layer ? m : 2m) adjacency rows in
 * the same order, holding point ids, ANN_NONE padded.  Blocks.               */
int ann_hnsw_copy_layer(const ann_hnsw* h, uint32_t layer, uint32_t* ids_host, uint32_t* rows_host);
/* Counters of one layer (the beam-1 passes of points that do not belong to
 * the layer count as searches of it).                                        */
int ann_hnsw_get_stats(const ann_hnsw* h, uint32_t layer, ann_stats* stats);
void ann_hnsw_free(ann_hnsw* h);

/* ------------------------------------------------------------------------
 * Clustering-based builder (Sec. 3.2 and 4.3, ParlayHCNNG).  T cluster trees;
 * a node with more than Ls points is split by two pivots drawn among its
 * points (a point goes with the pivot it is nearer to, the first on ties);
 * in every leaf a spanning tree is grown by Kruskal's scan over the pairs
 * (point, one of its l nearest neighbours in the leaf), no point taking more
 * than s tree edges; a point's row is prune(p, its tree neighbours over all
 * trees, R) with the alpha rule of Sec. 4.1.
 *   random numbers   draw(tree, node, j) = the (k+1)-th output of
 *                    SplitMix64(seed), k = 2 * (tree * 2^40 + node) + j,
 *                    nodes numbered like a binary heap (root 1)
 *   pivots           a node holds its c points in ascending id order; the
 *                    pivots stand at positions mulhi64(draw(..,0), c) and
 *                    mulhi64(draw(..,1), c - 1), the second moved up by one
 *                    when it is not below the first
 *   degenerate cut   when one side stays empty, or at depth 39, the node's
 *                    order is cut in the middle (ceil(c/2) points left)
 *   pairs            sorted by (distance, smaller id, larger id)
 * The result is a graph like ann_build's (start vertex = ann_start_vertex);
 * ann_search and ann_search_eps serve it.
 *   ANN_U8 / ANN_I8 with ANN_L2SQ and d <= 128 (exact integers throughout), or
 *   ANN_F32 with either metric, d % 4 == 0 and d <= 256 (fp32 sums on the
 *   vector units and the fp32 matrix cores; squared L2 inside a leaf is taken
 *   as |a|^2 + |b|^2 - 2<a,b> to pick a point's l candidates, whose distances
 *   are then taken again as sum (a - b)^2);
 *   1 <= T < 2^20, 2 <= Ls <= 1024, 1 <= l <= 16, Ls * l <= 16384,
 *   1 <= s <= 255, 1 <= R <= 512, T * 2n < 2^32.
 * Blocks until done.
 * Test-only option: with ANN_HCNNG_FEW_TILES set in the environment the
 * buffer of leaf tiles starts with room for one tile, so that every build
 * takes the path that allocates it again at the size a group of trees needs
 * (otherwise reached only by inputs that split into very many tiny leaves).
 * The result does not depend on it.
 * ------------------------------------------------------------------------ */
int ann_hcnng_build(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                    uint32_t T, uint32_t Ls, uint32_t s, uint32_t l, uint32_t R, float alpha, uint64_t seed,
                    void* stream, ann_graph** out);

/* One cluster tree and its leaves' spanning trees alone (for tests): perm_host
 * receives the n point ids leaf after leaf, leaf_off_host the *nleaves + 1
 * leaf boundaries (room for n + 1), pairs_host the accepted pairs (two ids
 * each, room for n pairs) leaf after leaf in the order they were accepted.   */
int ann_hcnng_tree_edges(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                         uint32_t Ls, uint32_t s, uint32_t l, uint64_t seed, uint32_t tree, void* stream,
                         uint32_t* perm_host, uint64_t* leaf_off_host, uint64_t* nleaves,
                         uint32_t* pairs_host, uint64_t* npairs);

/* The nearest neighbours inside the leaves of one cluster tree, as the builder's
 * kernels computed them before the pairs are sorted (for tests of Sec. 4.3's
 * "l nearest neighbours in the leaf"): perm_host / leaf_off_host / nleaves as in
 * ann_hcnng_tree_edges; knn_ids_host receives n x l point ids, row i for the
 * point perm_host[i], nearest first by (distance, position in the leaf),
 * ANN_NONE where the leaf has fewer other points; knn_dists_host the n x l
 * distances (int32 for u8/i8, float for f32; INT32_MAX / +inf padding).       */
int ann_hcnng_leaf_knn(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                       uint32_t Ls, uint32_t l, uint64_t seed, uint32_t tree, void* stream, uint32_t* perm_host,
                       uint64_t* leaf_off_host, uint64_t* nleaves, uint32_t* knn_ids_host, void* knn_dists_host);

/* Thread-local description of the last error on this thread ("" if none).   */
const char* ann_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
