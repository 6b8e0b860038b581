/*
 * hnsw_oracle.h -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain CPU statement of the layered index of Sec. 4.2 (ParlayHNSW): a
 * hierarchy of graphs in which layer l holds the points whose level is at
 * least l, every layer built with the prefix-doubling batch insertion of
 * Alg. 3 (one batch insertion per layer), searched from the top with a
 * beam of one down to layer 1 and with the full beam on layer 0.  It is
 * built on the primitives of vamana_oracle.h (greedy search, prune,
 * BatchInsert) and, like them, shares no code with the HIP library.
 *
 * What the paper leaves open, as read here (the HIP library implements the
 * same readings separately; the tests compare the two):
 *   - level of point i: with r = the (i+1)-th output of SplitMix64(seed),
 *     the largest l such that r <= floor((2^64 - 1) / m^l): a geometric
 *     law of ratio 1/m, the rule of the published HNSW algorithm
 *     (floor(-ln(u) / ln(m))) in integers;
 *   - degree bounds: m on the layers above the bottom, 2m at the bottom
 *     (appendix, parameter paragraph);
 *   - entry point: the point of the highest level, smallest id on ties; it
 *     is in every layer from the beginning with empty rows and is never
 *     inserted (the role the start vertex has in vamana_oracle.h);
 *   - insertion order and batch sizes: those of vo_build with the entry
 *     point in place of the start vertex;
 *   - a batch point of level lv walks down from the entry point: on every
 *     layer above lv a search with beam 1 over that layer as it stood
 *     before the batch, its result being the start vertex one layer
 *     below; on the layers lv..0 BatchInsert with beam efc from that start
 *     vertex, the vertex closest to the point among those the search
 *     visited being the start vertex one layer below;
 *   - prune is the alpha rule of Sec. 4.1 on every layer (none of the
 *     further heuristics of the original);
 *   - a query walks down the same way (beam 1 on layers top..1) and then
 *     runs the search of Alg. 1, with the (1 + eps) rule if asked, on
 *     layer 0.
 *
 * Parity pins (tests/test_oracle_hnsw.py): levels against a re-statement in
 * Python integers and their geometric law; a build with every level zero
 * against vo_build with R = 2m; a build with batches of one against Alg. 2
 * applied layer by layer from Python; layer invariants; a search worked by
 * hand on a hand-made three-layer index.
 */
#ifndef HNSW_ORACLE_H
#define HNSW_ORACLE_H

#include "vamana_oracle.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  uint64_t n;
  uint32_t m;      /* degree bound of the layers above the bottom; bottom: 2m */
  uint32_t top;    /* highest layer                                           */
  uint32_t entry;  /* entry point, a point of layer `top`                     */
  uint32_t* level; /* n                                                       */
  uint32_t** rows; /* top+1 arrays; rows[l] is n x (l ? m : 2m), VO_NONE
                      padded; rows of points below layer l are all VO_NONE    */
} vo_hnsw;

uint32_t vo_hnsw_level(uint64_t seed, uint32_t id, uint32_t m);

/* Builds the index.  `level` (n entries) and `order` (n-1 ids, the entry
 * point left out) may be NULL: then they are drawn from `seed`.  theta = 0
 * means max(1, n/50).  max_rounds = 0 runs every batch.                     */
int vo_hnsw_build(const vo_data* data, uint32_t m, uint32_t efc, double alpha, uint64_t seed,
                  uint64_t theta, const uint32_t* level, const uint32_t* order,
                  uint64_t max_rounds, int threads, vo_hnsw** out, vo_stats* stats);

/* One batch (what vo_hnsw_build does per round): the b points of `batch`,
 * none of them in the index yet, walk down and are inserted as described
 * above.  Their levels are read from h->level.                              */
int vo_hnsw_insert_batch(const vo_data* data, vo_hnsw* h, const uint32_t* batch, uint64_t b,
                         uint32_t efc, double alpha, int threads, vo_stats* stats);

void vo_hnsw_free(vo_hnsw* h);

/* Queries.  ids_out nq x k, dists_out as vo_search_batch (may be NULL);
 * entry_out (may be NULL) receives the start vertex each query reached for
 * layer 0.  eps < 0: no (1 + eps) rule.                                     */
int vo_hnsw_search_batch(const vo_data* data, const vo_hnsw* h, const void* queries, uint64_t nq,
                         uint32_t k, uint32_t L, double eps, int threads, uint32_t* ids_out,
                         void* dists_out, uint32_t* entry_out, vo_stats* stats);

#ifdef __cplusplus
}
#endif
#endif
