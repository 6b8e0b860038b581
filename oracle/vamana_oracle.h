/*
 * vamana_oracle.h -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, sequential CPU statement of what the GPU hot path must
 * compute: greedy beam search (Alg. 1 of the paper), sequential insertion
 * (Alg. 2), prefix-doubling batch insertion (Alg. 3) and the alpha-prune rule
 * of Sec. 4.1, for a Vamana/DiskANN-style graph.  It shares no code with the
 * HIP library and must never be linked, imported or called by it.  Only the
 * tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * All pointers are host pointers.  Points and queries are row-major n x d
 * arrays of the given dtype.  A graph is n x R uint32 rows; valid neighbours
 * come first in a row and unused slots hold VO_NONE.
 *
 * Conventions the paper leaves open (each one also implemented, separately,
 * by the HIP library; the tests compare the two):
 *   - every "closest" is taken under the total order (distance, id);
 *   - distances: u8/i8 squared L2 is the exact integer; f32 squared L2 and
 *     f32 negative inner product are accumulated in double, rounded once to
 *     float, and +0.0f is added so that -0 becomes +0;
 *   - the alpha test on integers is  a16 * d(p*,p') <= d(p,p') * 65536  with
 *     a16 = llround(alpha * 65536), in 64-bit integers; on f32 it is the
 *     single-precision product  (float)alpha * d(p*,p') <= d(p,p');
 *   - start vertex = point nearest (squared L2) to the mean, smallest id on
 *     ties; it is present from the beginning with an empty row and is never
 *     re-inserted;
 *   - insertion order = Fisher-Yates shuffle, from the front, of the ids other
 *     than the start vertex in ascending order: step i = 0..m-2 exchanges
 *     positions i and i + mulhi64(r, m - i), r the next output of
 *     SplitMix64(seed) (position i is final after step i);
 *   - batch sizes: with `done` points already taken from the order and
 *     m = n-1 in total, the next batch has  min(done+2, theta, m-done)
 *     points, i.e. 2,4,8,... capped by theta (Alg. 3 with the batch size,
 *     not the end index, bounded by theta as the text of Sec. 3.1 says);
 *   - reverse edges of one destination are appended in batch order.
 *
 * Parity pins (tests/test_oracle_*.py): distances against integer closed
 * forms and numpy; beam search against brute force on complete graphs, BFS
 * closure when L >= n, and a hand-worked path graph; prune against top-R
 * (huge alpha), single neighbour (tiny alpha), a hand-worked 1-D example and
 * an independent audit of every kept/dropped candidate; the schedule against
 * its closed form; batch insertion with every batch of size one against
 * Alg. 2; a hand-worked five-point build; degree and snapshot invariants;
 * streaming insertion against the one-shot build whose batches it continues
 * and, with theta = 1, against Alg. 2 point by point.
 */
#ifndef VAMANA_ORACLE_H
#define VAMANA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VO_NONE 0xFFFFFFFFu

enum { VO_U8 = 0, VO_I8 = 1, VO_F32 = 2 };
enum { VO_L2SQ = 0, VO_MIPS = 1 };

typedef struct {
  const void* points; /* n x d, row-major                         */
  uint64_t n;
  uint32_t d;
  int dtype;  /* VO_U8 / VO_I8 / VO_F32                            */
  int metric; /* VO_L2SQ / VO_MIPS (MIPS: distance = -<a,b>)       */
} vo_data;

typedef struct {
  uint64_t searches;   /* greedy searches run                       */
  uint64_t hops;       /* vertices processed (|V| summed)           */
  uint64_t evals;      /* distinct vertices whose distance was taken */
  uint64_t prunes;     /* prune calls in step 1                     */
  uint64_t reprunes;   /* prune calls in step 2 (overflowing rows)  */
  uint64_t appends;    /* destinations that only appended           */
  uint64_t edges;      /* reverse edges grouped                     */
  uint64_t prune_cand; /* candidates handed to all prune calls      */
  uint64_t prune_evals;/* pair distances taken inside prune         */
  uint64_t rounds;
} vo_stats;

/* Distance between two vectors of `d` elements of `dtype`.  Returned as a
 * double holding the exact integer (u8/i8) or the rounded float (f32).     */
double vo_distance(const void* a, const void* b, uint32_t d, int dtype, int metric);

/* Alg. 1.  `graph` n x R.  `query` = d elements of data->dtype.
 * V (processing order) goes to v_ids/v_dists (capacity v_cap; *nv receives
 * the true count even if it exceeds v_cap), the k closest to k_ids/k_dists
 * (padded with VO_NONE / +inf).  Returns 0, or -1 on bad arguments.        */
int vo_greedy_search(const vo_data* data, const uint32_t* graph, uint32_t R,
                     uint32_t start, const void* query, uint32_t L, uint32_t k,
                     uint32_t* v_ids, double* v_dists, uint64_t v_cap, uint64_t* nv,
                     uint32_t* k_ids, double* k_dists, vo_stats* stats);

/* The same with the (1 + eps) rule of Sec. 4.5: a vertex is searched only while its distance is
 * within the factor 1 + eps of the current k-th nearest candidate (squared distances for L2;
 * the bound is dk + eps * |dk|).  eps < 0 switches the rule off; eps must be below 16384.     */
int vo_greedy_search_eps(const vo_data* data, const uint32_t* graph, uint32_t R,
                         uint32_t start, const void* query, uint32_t L, uint32_t k, double eps,
                         uint32_t* v_ids, double* v_dists, uint64_t v_cap, uint64_t* nv,
                         uint32_t* k_ids, double* k_dists, vo_stats* stats);

/* prune(p, C, R) of Sec. 4.1: `p_vec` is the vector of p, `p_id` its id
 * (removed from C; VO_NONE if p is not a member of the data set).  `cand`
 * holds m ids (duplicates allowed).  Writes the selected ids, in selection
 * order, to out[0..R) padded with VO_NONE and returns their count.         */
uint32_t vo_prune(const vo_data* data, const void* p_vec, uint32_t p_id,
                  const uint32_t* cand, uint64_t m, uint32_t R, double alpha,
                  uint32_t* out, vo_stats* stats);

/* Start vertex: argmin_i ||x_i - mean||^2, ties to the smaller id.         */
uint32_t vo_start_vertex(const vo_data* data);

/* Insertion order: writes the n-1 ids other than `start`.                  */
void vo_insertion_order(uint64_t n, uint32_t start, uint64_t seed, uint32_t* order);

/* Batch boundaries over m = n-1 ordered points: bounds[0]=0 < ... <
 * bounds[rounds]=m.  Returns the number of rounds (bounds may be NULL to
 * count only; otherwise it must hold rounds+1 entries).                    */
uint64_t vo_schedule(uint64_t m, uint64_t theta, uint64_t* bounds);

/* Alg. 2: insert point `p` into `graph` (n x R, modified in place).        */
int vo_insert(const vo_data* data, uint32_t* graph, uint32_t R, uint32_t start,
              uint32_t p, uint32_t L, double alpha, vo_stats* stats);

/* BatchInsert of Alg. 3 for the ids batch[0..b).  `threads` > 1 runs the two
 * parallel-for loops of the listing with OpenMP (same result as 1).        */
int vo_batch_insert(const vo_data* data, uint32_t* graph, uint32_t R, uint32_t start,
                    const uint32_t* batch, uint64_t b, uint32_t L, double alpha,
                    int threads, vo_stats* stats);

/* The same with a start vertex of its own for every batch point (starts[i],
 * or `start` for all when starts is NULL); nearest_out[i], when given,
 * receives the vertex closest to batch[i] among those its search visited.
 * This is the form the layers of an HNSW index need (hnsw_oracle.h).       */
int vo_batch_insert_from(const vo_data* data, uint32_t* graph, uint32_t R, uint32_t start,
                         const uint32_t* starts, const uint32_t* batch, uint64_t b, uint32_t L,
                         double alpha, int threads, uint32_t* nearest_out, vo_stats* stats);

/* Alg. 3: whole build.  `order` (n-1 ids) may be NULL: then it is drawn from
 * `seed`.  `start` may be VO_NONE: then vo_start_vertex is used.  theta = 0
 * means max(1, n/50).  `graph` receives n x R.  max_rounds = 0 runs all
 * rounds, otherwise stops after that many (for per-round checks).          */
int vo_build(const vo_data* data, uint32_t R, uint32_t L, double alpha, uint64_t seed,
             uint64_t theta, uint32_t start, const uint32_t* order, uint64_t max_rounds,
             int threads, uint32_t* graph, uint32_t* start_out, vo_stats* stats);

/* Streaming insertion of the points n_old..n-1 (n = data->n) into a graph
 * that holds the points 0..n_old-1: `graph` is n x R, rows of the new ids
 * all VO_NONE on entry.  The new ids are taken in `order` (n - n_old ids,
 * each new id once) or, when it is NULL, in the order vo_new_points_order
 * draws from `seed`; they are inserted with BatchInsert of Alg. 3 in batches
 * of min(present + 2, theta, left) points, `present` counting the points
 * other than the start vertex that the graph holds at that moment: the
 * schedule of vo_build carried on.  theta = 0 means max(1, n/50).  The start
 * vertex stays what it was.                                                 */
int vo_insert_points(const vo_data* data, uint32_t* graph, uint32_t R, uint32_t start,
                     uint64_t n_old, uint32_t L, double alpha, uint64_t seed, uint64_t theta,
                     const uint32_t* order, uint64_t max_rounds, int threads, vo_stats* stats);

/* The ids first..first+count-1 shuffled like vo_insertion_order shuffles
 * the ids of a build (Fisher-Yates from the front, SplitMix64(seed)).        */
void vo_new_points_order(uint64_t first, uint64_t count, uint64_t seed, uint32_t* order);

/* vo_schedule for m further points when `present` are already in: bounds[0]
 * = 0 < ... < bounds[rounds] = m, relative to the first new point.          */
uint64_t vo_schedule_from(uint64_t present, uint64_t m, uint64_t theta, uint64_t* bounds);

/* Sequential build: Alg. 2 applied to every id of the order, one by one.   */
int vo_build_sequential(const vo_data* data, uint32_t R, uint32_t L, double alpha,
                        uint32_t start, const uint32_t* order, uint64_t m, uint32_t* graph,
                        vo_stats* stats);

/* Batched queries: greedySearch(q, start, L, k) for each of nq queries.
 * dists_out is int32[nq*k] for u8/i8 and float[nq*k] for f32; padding is
 * VO_NONE with INT32_MAX / +inf.                                           */
int vo_search_batch(const vo_data* data, const uint32_t* graph, uint32_t R, uint32_t start,
                    const void* queries, uint64_t nq, uint32_t k, uint32_t L, int threads,
                    uint32_t* ids_out, void* dists_out, vo_stats* stats);
int vo_search_batch_eps(const vo_data* data, const uint32_t* graph, uint32_t R, uint32_t start,
                        const void* queries, uint64_t nq, uint32_t k, uint32_t L, double eps,
                        int threads, uint32_t* ids_out, void* dists_out, vo_stats* stats);

/* The same with a start vertex of its own for every query (starts[q]; NULL:
 * `start` for all); dists_out may be NULL.                                  */
int vo_search_batch_from(const vo_data* data, const uint32_t* graph, uint32_t R, uint32_t start,
                         const uint32_t* starts, const void* queries, uint64_t nq, uint32_t k,
                         uint32_t L, double eps, int threads, uint32_t* ids_out, void* dists_out,
                         vo_stats* stats);

/* Exact k nearest neighbours by exhaustive scan under (distance, id).      */
int vo_brute_force(const vo_data* data, const void* queries, uint64_t nq, uint32_t k,
                   int threads, uint32_t* ids_out, void* dists_out);

/* Number of OpenMP threads a `threads` argument resolves to (0 = all).     */
int vo_threads(int threads);

#ifdef __cplusplus
}
#endif
#endif
