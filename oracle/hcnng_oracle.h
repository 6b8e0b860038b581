/*
 * hcnng_oracle.h -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain CPU statement of the clustering-based builder of Sec. 4.3
 * (ParlayHCNNG) with the cluster trees of Sec. 3.2: T random cluster trees;
 * in every leaf a degree-bounded minimum spanning tree over the graph that
 * joins each point to its l nearest neighbours inside the leaf (a spanning
 * tree restricted to those edges); the union of all leaves' edges, pruned
 * per point with the alpha rule of Sec. 4.1.  Built on vo_distance and vo_prune of
 * vamana_oracle.h; shares no code with the HIP library.
 *
 * What the paper leaves open, as read here (the HIP library implements the
 * same readings separately; the tests compare the two):
 *   - random numbers: draw(tree, node, j) = the (k+1)-th output of
 *     SplitMix64(seed), k = 2 * (tree * 2^40 + node) + j; nodes are numbered
 *     like a binary heap (root 1, children 2v and 2v+1);
 *   - a node holds its points in ascending id order (the root holds all);
 *     with c points, the two pivots are the points at positions
 *     i1 = mulhi64(draw(..,0), c) and i2 = mulhi64(draw(..,1), c-1), i2
 *     moved up by one when i2 >= i1 (two distinct positions);
 *   - a point goes left when it is at most as far from the first pivot as
 *     from the second, right otherwise; if one side stays empty (equal
 *     points), or at depth 39, the node is cut in the middle of its order
 *     instead (the first ceil(c/2) points left);
 *   - a node of at most Ls points is a leaf;
 *   - inside a leaf every point takes its min(l, c-1) nearest other points
 *     under (distance, id); the undirected pairs so formed, each once, are
 *     sorted by (distance, smaller id, larger id) and scanned in that order:
 *     a pair joins the tree when its ends lie in different components and
 *     both have fewer than s tree edges (Kruskal with a degree bound);
 *   - the neighbours of a point are the other ends of its tree edges over
 *     all T trees, each once; its row is prune(p, neighbours, R) with the
 *     alpha rule, applied whether or not there are more than R.
 *
 * Parity pins (tests/test_oracle_hcnng.py): the cluster tree against a
 * re-statement in Python; leaf trees against scipy's minimum spanning tree
 * when neither l nor s restricts, against a Python re-statement when they
 * do, and a hand-worked example where the degree bound bites; the rows of a
 * whole build against the prune audit over the union of the re-stated
 * leaves' edges.
 */
#ifndef HCNNG_ORACLE_H
#define HCNNG_ORACLE_H

#include "vamana_oracle.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One cluster tree: perm receives the n point ids leaf after leaf (ascending
 * inside a leaf), leaf_off the nleaves+1 boundaries (room for n+1 entries). */
int vo_hcnng_tree(const vo_data* data, uint32_t Ls, uint64_t seed, uint32_t tree, uint32_t* perm,
                  uint64_t* leaf_off, uint64_t* nleaves);

/* The degree-bounded tree of one leaf: ids (cnt of them, ascending); eu/ev
 * (room for cnt-1 each) receive the accepted pairs in the order they were
 * accepted, eu < ev.  Returns their number in *ne.                          */
int vo_hcnng_leaf(const vo_data* data, const uint32_t* ids, uint32_t cnt, uint32_t s, uint32_t l,
                  uint32_t* eu, uint32_t* ev, uint64_t* ne);

typedef struct {
  uint64_t leaves;      /* over all trees                          */
  uint64_t tree_edges;  /* accepted pairs over all trees           */
  uint64_t neighbours;  /* distinct (point, neighbour) before prune */
} vo_hcnng_stats;

/* The whole build; graph receives n x R rows (VO_NONE padded).             */
int vo_hcnng_build(const vo_data* data, uint32_t T, uint32_t Ls, uint32_t s, uint32_t l, uint32_t R,
                   double alpha, uint64_t seed, int threads, uint32_t* graph, vo_hcnng_stats* stats);

#ifdef __cplusplus
}
#endif
#endif
