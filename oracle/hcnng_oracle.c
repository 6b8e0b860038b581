/*
 * hcnng_oracle.c -- TEST INFRASTRUCTURE, not product code.  See hcnng_oracle.h.
 */
#include "hcnng_oracle.h"

#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static size_t elem_bytes(int dtype) { return dtype == VO_F32 ? 4 : 1; }

static const void* vec_of(const vo_data* D, uint32_t id) {
  return (const char*)D->points + (size_t)id * D->d * elem_bytes(D->dtype);
}

static double dist_ids(const vo_data* D, uint32_t a, uint32_t b) {
  return vo_distance(vec_of(D, a), vec_of(D, b), D->d, D->dtype, D->metric);
}

/* the (k+1)-th output of SplitMix64(seed) */
static uint64_t stream_output(uint64_t seed, uint64_t k) {
  uint64_t z = seed + (k + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static uint64_t draw(uint64_t seed, uint32_t tree, uint64_t node, uint32_t j) {
  return stream_output(seed, 2 * (((uint64_t)tree << 40) + node) + j);
}

static uint64_t mulhi64(uint64_t a, uint64_t b) {
  return (uint64_t)(((unsigned __int128)a * (unsigned __int128)b) >> 64);
}

/* ------------------------------------------------------------------ */
/* cluster tree (Sec. 3.2, Sec. 4.3)                                    */
/* ------------------------------------------------------------------ */

typedef struct {
  const vo_data* D;
  uint32_t Ls;
  uint64_t seed;
  uint32_t tree;
  uint32_t* perm;     /* output, filled leaf after leaf */
  uint64_t* leaf_off; /* output                          */
  uint64_t nleaves;
  uint64_t filled;
  uint32_t* tmp;      /* n ids of scratch                */
} tree_ctx;

/* `ids` holds the node's c points in ascending order and is used as scratch below. */
static void split(tree_ctx* X, uint32_t* ids, uint64_t c, uint64_t node, uint32_t depth) {
  if (c <= X->Ls) {
    X->leaf_off[X->nleaves++] = X->filled;
    memcpy(X->perm + X->filled, ids, c * sizeof(uint32_t));
    X->filled += c;
    return;
  }
  uint64_t i1 = mulhi64(draw(X->seed, X->tree, node, 0), c);
  uint64_t i2 = mulhi64(draw(X->seed, X->tree, node, 1), c - 1);
  if (i2 >= i1) ++i2;
  uint32_t p1 = ids[i1], p2 = ids[i2];
  uint64_t nl = 0, nr = 0;
  uint32_t* right = X->tmp; /* right side parked here while the left side is compacted in place */
  if (depth < 39) {
    for (uint64_t i = 0; i < c; ++i) {
      uint32_t x = ids[i];
      if (dist_ids(X->D, x, p1) <= dist_ids(X->D, x, p2))
        ids[nl++] = x;
      else
        right[nr++] = x;
    }
  }
  if (nl == 0 || nr == 0) {
    /* nothing separated (or the tree is too deep): cut the order in the middle */
    if (depth < 39 && nr > 0) memcpy(ids, right, nr * sizeof(uint32_t)); /* nl == 0: all went right */
    nl = (c + 1) / 2;
    nr = c - nl;
  } else {
    memcpy(ids + nl, right, nr * sizeof(uint32_t));
  }
  split(X, ids, nl, 2 * node, depth + 1);
  split(X, ids + nl, nr, 2 * node + 1, depth + 1);
}

int vo_hcnng_tree(const vo_data* D, uint32_t Ls, uint64_t seed, uint32_t tree, uint32_t* perm,
                  uint64_t* leaf_off, uint64_t* nleaves) {
  if (!D || !perm || !leaf_off || !nleaves || D->n < 1 || Ls < 2 || tree >= (1u << 20)) return -1;
  uint64_t n = D->n;
  uint32_t* ids = (uint32_t*)malloc(n * sizeof(uint32_t));
  uint32_t* tmp = (uint32_t*)malloc(n * sizeof(uint32_t));
  if (!ids || !tmp) {
    free(ids);
    free(tmp);
    return -1;
  }
  for (uint64_t i = 0; i < n; ++i) ids[i] = (uint32_t)i;
  tree_ctx X;
  X.D = D;
  X.Ls = Ls;
  X.seed = seed;
  X.tree = tree;
  X.perm = perm;
  X.leaf_off = leaf_off;
  X.nleaves = 0;
  X.filled = 0;
  X.tmp = tmp;
  split(&X, ids, n, 1, 0);
  leaf_off[X.nleaves] = n;
  *nleaves = X.nleaves;
  free(ids);
  free(tmp);
  return 0;
}

/* ------------------------------------------------------------------ */
/* one leaf: l nearest neighbours, then Kruskal with a degree bound     */
/* ------------------------------------------------------------------ */

typedef struct {
  double dist;
  uint32_t u, v; /* u < v */
} pair_t;

static int pair_cmp(const void* pa, const void* pb) {
  const pair_t* a = (const pair_t*)pa;
  const pair_t* b = (const pair_t*)pb;
  if (a->dist != b->dist) return a->dist < b->dist ? -1 : 1;
  if (a->u != b->u) return a->u < b->u ? -1 : 1;
  if (a->v != b->v) return a->v < b->v ? -1 : 1;
  return 0;
}

typedef struct {
  double dist;
  uint32_t id;
} near_t;

static int near_cmp(const void* pa, const void* pb) {
  const near_t* a = (const near_t*)pa;
  const near_t* b = (const near_t*)pb;
  if (a->dist != b->dist) return a->dist < b->dist ? -1 : 1;
  return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

static uint32_t uf_find(uint32_t* parent, uint32_t x) {
  while (parent[x] != x) x = parent[x];
  return x;
}

int vo_hcnng_leaf(const vo_data* D, const uint32_t* ids, uint32_t cnt, uint32_t s, uint32_t l,
                  uint32_t* eu, uint32_t* ev, uint64_t* ne) {
  if (!D || !ids || !ne) return -1;
  *ne = 0;
  if (cnt < 2) return 0;
  uint32_t k = l < cnt - 1 ? l : cnt - 1;
  near_t* row = (near_t*)malloc((size_t)cnt * sizeof(near_t));
  pair_t* pairs = (pair_t*)malloc((size_t)cnt * k * sizeof(pair_t));
  uint32_t* parent = (uint32_t*)malloc(cnt * sizeof(uint32_t));
  uint32_t* deg = (uint32_t*)calloc(cnt, sizeof(uint32_t));
  if (!row || !pairs || !parent || !deg) {
    free(row);
    free(pairs);
    free(parent);
    free(deg);
    return -1;
  }
  /* the k nearest other points of every point, positions in `ids` standing for the points
   * (ids ascend, so position order is id order) */
  uint64_t np = 0;
  for (uint32_t a = 0; a < cnt; ++a) {
    uint32_t m = 0;
    for (uint32_t b = 0; b < cnt; ++b) {
      if (b == a) continue;
      row[m].dist = dist_ids(D, ids[a], ids[b]);
      row[m].id = b;
      ++m;
    }
    qsort(row, m, sizeof(near_t), near_cmp);
    for (uint32_t j = 0; j < k; ++j) {
      pairs[np].dist = row[j].dist;
      pairs[np].u = a < row[j].id ? a : row[j].id;
      pairs[np].v = a < row[j].id ? row[j].id : a;
      ++np;
    }
  }
  qsort(pairs, np, sizeof(pair_t), pair_cmp);
  for (uint32_t i = 0; i < cnt; ++i) parent[i] = i;
  uint64_t out = 0;
  for (uint64_t i = 0; i < np; ++i) {
    if (i > 0 && pairs[i].u == pairs[i - 1].u && pairs[i].v == pairs[i - 1].v) continue; /* each pair once */
    uint32_t u = pairs[i].u, v = pairs[i].v;
    if (deg[u] >= s || deg[v] >= s) continue;
    uint32_t ru = uf_find(parent, u), rv = uf_find(parent, v);
    if (ru == rv) continue;
    parent[ru] = rv;
    ++deg[u];
    ++deg[v];
    if (eu) eu[out] = ids[u];
    if (ev) ev[out] = ids[v];
    ++out;
  }
  *ne = out;
  free(row);
  free(pairs);
  free(parent);
  free(deg);
  return 0;
}

/* ------------------------------------------------------------------ */
/* the whole build                                                      */
/* ------------------------------------------------------------------ */

typedef struct {
  uint32_t p, q;
} arc_t;

static int arc_cmp(const void* pa, const void* pb) {
  const arc_t* a = (const arc_t*)pa;
  const arc_t* b = (const arc_t*)pb;
  if (a->p != b->p) return a->p < b->p ? -1 : 1;
  return a->q < b->q ? -1 : (a->q > b->q ? 1 : 0);
}

int vo_hcnng_build(const vo_data* D, uint32_t T, uint32_t Ls, uint32_t s, uint32_t l, uint32_t R,
                   double alpha, uint64_t seed, int threads, uint32_t* graph, vo_hcnng_stats* stats) {
  if (!D || !graph || D->n < 1 || T < 1 || Ls < 2 || s < 1 || l < 1 || R < 1) return -1;
  uint64_t n = D->n;
  int nthreads = vo_threads(threads);
  (void)nthreads;
  vo_hcnng_stats st;
  memset(&st, 0, sizeof(st));
  /* every tree yields at most n-1 pairs, i.e. 2(n-1) arcs */
  arc_t* arcs = (arc_t*)malloc((size_t)T * 2 * n * sizeof(arc_t));
  uint32_t* perm = (uint32_t*)malloc(n * sizeof(uint32_t));
  uint64_t* off = (uint64_t*)malloc((n + 1) * sizeof(uint64_t));
  uint32_t* eu = (uint32_t*)malloc(n * sizeof(uint32_t));
  uint32_t* ev = (uint32_t*)malloc(n * sizeof(uint32_t));
  uint64_t* eoff = (uint64_t*)malloc((n + 1) * sizeof(uint64_t));
  if (!arcs || !perm || !off || !eu || !ev || !eoff) {
    free(arcs);
    free(perm);
    free(off);
    free(eu);
    free(ev);
    free(eoff);
    return -1;
  }
  uint64_t na = 0;
  int err = 0;
  for (uint32_t t = 0; t < T && !err; ++t) {
    uint64_t nleaves = 0;
    if (vo_hcnng_tree(D, Ls, seed, t, perm, off, &nleaves)) {
      err = -1;
      break;
    }
    st.leaves += nleaves;
    /* leaf j writes its pairs at eu/ev + (off[j] - j): a leaf of c points has at most c-1 */
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t j = 0; j < (int64_t)nleaves; ++j) {
      uint64_t ne = 0;
      uint64_t base = off[j] - (uint64_t)j;
      if (vo_hcnng_leaf(D, perm + off[j], (uint32_t)(off[j + 1] - off[j]), s, l, eu + base, ev + base, &ne))
        err = -1;
      eoff[j] = ne;
    }
    for (uint64_t j = 0; j < nleaves && !err; ++j) {
      uint64_t base = off[j] - j;
      for (uint64_t e = 0; e < eoff[j]; ++e) {
        arcs[na].p = eu[base + e];
        arcs[na].q = ev[base + e];
        ++na;
        arcs[na].p = ev[base + e];
        arcs[na].q = eu[base + e];
        ++na;
      }
      st.tree_edges += eoff[j];
    }
  }
  if (!err) {
    qsort(arcs, na, sizeof(arc_t), arc_cmp);
    memset(graph, 0xFF, (size_t)n * R * sizeof(uint32_t));
    /* boundaries of every point's arcs */
    uint64_t* first = (uint64_t*)malloc((n + 1) * sizeof(uint64_t));
    uint64_t a = 0;
    for (uint64_t p = 0; p < n; ++p) {
      first[p] = a;
      while (a < na && arcs[a].p == p) ++a;
    }
    first[n] = na;
    uint64_t distinct = 0;
#pragma omp parallel for schedule(dynamic, 256) num_threads(nthreads) reduction(+ : distinct)
    for (int64_t p = 0; p < (int64_t)n; ++p) {
      uint64_t lo = first[p], hi = first[p + 1];
      if (hi == lo) continue;
      uint32_t* cand = (uint32_t*)malloc((hi - lo) * sizeof(uint32_t));
      uint64_t c = 0;
      for (uint64_t i = lo; i < hi; ++i)
        if (i == lo || arcs[i].q != arcs[i - 1].q) cand[c++] = arcs[i].q;
      distinct += c;
      vo_prune(D, vec_of(D, (uint32_t)p), (uint32_t)p, cand, c, R, alpha, graph + (size_t)p * R, NULL);
      free(cand);
    }
    st.neighbours = distinct;
    free(first);
  }
  if (stats) *stats = st;
  free(arcs);
  free(perm);
  free(off);
  free(eu);
  free(ev);
  free(eoff);
  return err;
}
