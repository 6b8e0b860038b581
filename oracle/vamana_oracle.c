/*
 * vamana_oracle.c -- TEST INFRASTRUCTURE (see vamana_oracle.h).
 *
 * Sequential, deliberately plain.  Nothing is blocked, fused or reordered
 * beyond what the listings state; the only parallelism is an optional OpenMP
 * "parallel for" over exactly the two loops that Alg. 3 marks parallel (and
 * over independent queries), which cannot change the result because each
 * iteration reads only the frozen snapshot and writes only its own row.
 */
#include "vamana_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* small helpers                                                       */
/* ------------------------------------------------------------------ */

static size_t elem_size(int dtype) { return dtype == VO_F32 ? 4 : 1; }

static const void* row_ptr(const vo_data* D, uint64_t i) {
  return (const char*)D->points + (size_t)i * D->d * elem_size(D->dtype);
}

int vo_threads(int threads) {
#ifdef _OPENMP
  if (threads <= 0) return omp_get_max_threads();
  return threads;
#else
  (void)threads;
  return 1;
#endif
}

static void stats_add(vo_stats* into, const vo_stats* s) {
  if (!into) return;
  into->searches += s->searches;
  into->hops += s->hops;
  into->evals += s->evals;
  into->prunes += s->prunes;
  into->reprunes += s->reprunes;
  into->appends += s->appends;
  into->edges += s->edges;
  into->prune_cand += s->prune_cand;
  into->prune_evals += s->prune_evals;
  into->rounds += s->rounds;
}

/* ------------------------------------------------------------------ */
/* distances (Sec. 2: smaller is closer; Appendix A: TEXT2IMAGE uses    */
/* the negative inner product)                                          */
/* ------------------------------------------------------------------ */

double vo_distance(const void* a, const void* b, uint32_t d, int dtype, int metric) {
  if (dtype == VO_U8 || dtype == VO_I8) {
    int64_t acc = 0;
    for (uint32_t i = 0; i < d; ++i) {
      int64_t x, y;
      if (dtype == VO_U8) {
        x = ((const uint8_t*)a)[i];
        y = ((const uint8_t*)b)[i];
      } else {
        x = ((const int8_t*)a)[i];
        y = ((const int8_t*)b)[i];
      }
      if (metric == VO_L2SQ)
        acc += (x - y) * (x - y);
      else
        acc -= x * y;
    }
    return (double)acc;
  }
  const float* fa = (const float*)a;
  const float* fb = (const float*)b;
  double acc = 0.0;
  for (uint32_t i = 0; i < d; ++i) {
    double x = fa[i], y = fb[i];
    if (metric == VO_L2SQ)
      acc += (x - y) * (x - y);
    else
      acc -= x * y;
  }
  volatile float r = (float)acc; /* one rounding to single precision */
  r = r + 0.0f;                  /* -0 -> +0                         */
  return (double)r;
}

/* alpha * d(p*,p') <= d(p,p')  (Sec. 4.1) in the arithmetic stated in the
 * header: scaled 64-bit integers for u8/i8, one float product for f32.    */
static int alpha_dominates(int dtype, double alpha, double d_star_cand, double d_p_cand) {
  if (dtype == VO_U8 || dtype == VO_I8) {
    int64_t a16 = llround(alpha * 65536.0);
    int64_t lhs = a16 * (int64_t)d_star_cand;
    int64_t rhs = (int64_t)d_p_cand * 65536;
    return lhs <= rhs;
  }
  volatile float a = (float)alpha;
  volatile float prod = a * (float)d_star_cand;
  return prod <= (float)d_p_cand;
}

/* (1 + eps) rule of the search (Sec. 4.5): may a vertex at distance d be searched when the
 * k-th nearest candidate so far is at distance dk?  It may not if d exceeds dk by more than the
 * factor 1 + eps.  Integer distances: eps is quantised to e16 = round(eps * 2^16) and the test
 * is exact in 64-bit integers.  Floats: the bound is dk + eps * |dk| (which is (1 + eps) * dk for
 * dk >= 0 and stays meaningful for the negative values of the inner-product metric), one fp32
 * product and one fp32 sum.                                                              */
static int beyond_eps_bound(int dtype, double eps, double d, double dk) {
  if (dtype == VO_U8 || dtype == VO_I8) {
    int64_t e16 = llround(eps * 65536.0);
    return (int64_t)d * 65536 > (int64_t)dk * (65536 + e16);
  }
  volatile float e = (float)eps;
  volatile float prod = e * fabsf((float)dk);
  volatile float bound = (float)dk + prod;
  return (float)d > bound;
}

/* (distance, id) total order */
typedef struct {
  double dist;
  uint32_t id;
  uint32_t done; /* beam: already processed; prune: dead */
} cand_t;

static int cand_less(const cand_t* a, const cand_t* b) {
  if (a->dist != b->dist) return a->dist < b->dist;
  return a->id < b->id;
}

static int cand_cmp(const void* pa, const void* pb) {
  const cand_t* a = (const cand_t*)pa;
  const cand_t* b = (const cand_t*)pb;
  if (cand_less(a, b)) return -1;
  if (cand_less(b, a)) return 1;
  return 0;
}

/* ------------------------------------------------------------------ */
/* workspace: an exact "distance already taken" set (epoch stamps) and  */
/* the beam / visited arrays                                            */
/* ------------------------------------------------------------------ */

typedef struct {
  uint64_t n;
  uint32_t* stamp;
  uint32_t epoch;
  cand_t* beam; /* capacity L + R */
  uint64_t beam_cap;
  cand_t* vis;
  uint64_t vis_cap;
} work_t;

static int work_init(work_t* w, uint64_t n, uint32_t L, uint32_t R) {
  memset(w, 0, sizeof(*w));
  w->n = n;
  w->stamp = (uint32_t*)calloc(n ? n : 1, sizeof(uint32_t));
  w->beam_cap = (uint64_t)L + R + 1;
  w->beam = (cand_t*)malloc(w->beam_cap * sizeof(cand_t));
  w->vis_cap = 1024;
  w->vis = (cand_t*)malloc(w->vis_cap * sizeof(cand_t));
  if (!w->stamp || !w->beam || !w->vis) return -1;
  return 0;
}

static void work_free(work_t* w) {
  free(w->stamp);
  free(w->beam);
  free(w->vis);
  memset(w, 0, sizeof(*w));
}

static void work_new_search(work_t* w) {
  if (++w->epoch == 0) { /* wrapped: clear */
    memset(w->stamp, 0, w->n * sizeof(uint32_t));
    w->epoch = 1;
  }
}

/* ------------------------------------------------------------------ */
/* Alg. 1: greedySearch(q, s, L, k)                                     */
/* ------------------------------------------------------------------ */

/* Runs the search; on return w->vis[0..*nv) is V in processing order and
 * w->beam[0..*nbeam) the final beam, sorted.  Returns 0, -2 if the check
 * "k closest of V == first k of the beam" fails.                          */
static int greedy_core(const vo_data* D, const uint32_t* graph, uint32_t R, uint32_t start,
                       const void* query, uint32_t L, uint32_t k, double eps, work_t* w,
                       uint64_t* nv, uint64_t* nbeam, vo_stats* st) {
  work_new_search(w);
  uint64_t nb = 0, v = 0;
  w->beam[0].dist = vo_distance(query, row_ptr(D, start), D->d, D->dtype, D->metric);
  w->beam[0].id = start;
  w->beam[0].done = 0;
  nb = 1;
  w->stamp[start] = w->epoch;
  uint64_t evals = 1;

  for (;;) {
    /* p* = closest member of the beam not yet in V */
    uint64_t pi = nb;
    for (uint64_t i = 0; i < nb; ++i)
      if (!w->beam[i].done) {
        pi = i;
        break;
      }
    if (pi == nb) break;
    /* (1 + eps) rule, eps >= 0: only vertices within the bound of the current k-th nearest are
     * searched; the beam is sorted and the k-th distance never grows, so the first vertex that
     * fails ends the search */
    if (eps >= 0.0 && nb >= k && k >= 1 &&
        beyond_eps_bound(D->dtype, eps, w->beam[pi].dist, w->beam[k - 1].dist))
      break;
    w->beam[pi].done = 1;
    if (v == w->vis_cap) {
      w->vis_cap *= 2;
      w->vis = (cand_t*)realloc(w->vis, w->vis_cap * sizeof(cand_t));
      if (!w->vis) return -1;
    }
    w->vis[v++] = w->beam[pi];
    uint32_t pstar = w->beam[pi].id;

    /* beam <- beam U N_out(p*) */
    const uint32_t* row = graph + (size_t)pstar * R;
    for (uint32_t j = 0; j < R; ++j) {
      uint32_t x = row[j];
      if (x == VO_NONE) continue;
      if (w->stamp[x] == w->epoch) continue; /* distance already taken: it is in the
                                                beam, or was evicted and cannot return */
      w->stamp[x] = w->epoch;
      cand_t c;
      c.dist = vo_distance(query, row_ptr(D, x), D->d, D->dtype, D->metric);
      c.id = x;
      c.done = 0;
      ++evals;
      uint64_t pos = nb;
      while (pos > 0 && cand_less(&c, &w->beam[pos - 1])) {
        w->beam[pos] = w->beam[pos - 1];
        --pos;
      }
      w->beam[pos] = c;
      ++nb;
    }
    /* keep the L closest */
    if (nb > L) nb = L;
  }

  /* K from V must equal K from the beam (k <= L) */
  int rc = 0;
  {
    cand_t* sorted = (cand_t*)malloc((v ? v : 1) * sizeof(cand_t));
    if (!sorted) return -1;
    memcpy(sorted, w->vis, v * sizeof(cand_t));
    qsort(sorted, v, sizeof(cand_t), cand_cmp);
    uint64_t kk = k < nb ? k : nb;
    if (nb < k && v != nb) rc = -2;
    for (uint64_t i = 0; i < kk && rc == 0; ++i)
      if (sorted[i].id != w->beam[i].id || sorted[i].dist != w->beam[i].dist) rc = -2;
    free(sorted);
  }
  *nv = v;
  *nbeam = nb;
  if (st) {
    st->searches += 1;
    st->hops += v;
    st->evals += evals;
  }
  return rc;
}

int vo_greedy_search(const vo_data* D, const uint32_t* graph, uint32_t R, uint32_t start,
                     const void* query, uint32_t L, uint32_t k, uint32_t* v_ids,
                     double* v_dists, uint64_t v_cap, uint64_t* nv, uint32_t* k_ids,
                     double* k_dists, vo_stats* stats) {
  return vo_greedy_search_eps(D, graph, R, start, query, L, k, -1.0, v_ids, v_dists, v_cap, nv, k_ids,
                              k_dists, stats);
}

int vo_greedy_search_eps(const vo_data* D, const uint32_t* graph, uint32_t R, uint32_t start,
                         const void* query, uint32_t L, uint32_t k, double eps, uint32_t* v_ids,
                         double* v_dists, uint64_t v_cap, uint64_t* nv, uint32_t* k_ids,
                         double* k_dists, vo_stats* stats) {
  if (!D || !graph || !query || L < 1 || k > L || start >= D->n) return -1;
  if (!(eps < 16384.0)) return -1; /* keeps the integer form of the rule inside 64 bits */
  work_t w;
  if (work_init(&w, D->n, L, R)) {
    work_free(&w);
    return -1;
  }
  uint64_t v = 0, nb = 0;
  vo_stats st;
  memset(&st, 0, sizeof(st));
  int rc = greedy_core(D, graph, R, start, query, L, k, eps, &w, &v, &nb, &st);
  if (rc == 0 || rc == -2) {
    for (uint64_t i = 0; i < v && i < v_cap; ++i) {
      if (v_ids) v_ids[i] = w.vis[i].id;
      if (v_dists) v_dists[i] = w.vis[i].dist;
    }
    if (nv) *nv = v;
    for (uint32_t i = 0; i < k; ++i) {
      if (k_ids) k_ids[i] = i < nb ? w.beam[i].id : VO_NONE;
      if (k_dists) k_dists[i] = i < nb ? w.beam[i].dist : INFINITY;
    }
    stats_add(stats, &st);
  }
  work_free(&w);
  return rc;
}

/* ------------------------------------------------------------------ */
/* prune(p, C, R)  (Sec. 4.1)                                           */
/* ------------------------------------------------------------------ */

static int u32_cmp(const void* a, const void* b) {
  uint32_t x = *(const uint32_t*)a, y = *(const uint32_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

uint32_t vo_prune(const vo_data* D, const void* p_vec, uint32_t p_id, const uint32_t* cand,
                  uint64_t m, uint32_t R, double alpha, uint32_t* out, vo_stats* stats) {
  for (uint32_t i = 0; i < R; ++i) out[i] = VO_NONE;
  if (m == 0 || R == 0) return 0;

  /* C without p and without repeated ids */
  uint32_t* ids = (uint32_t*)malloc(m * sizeof(uint32_t));
  cand_t* c = (cand_t*)malloc(m * sizeof(cand_t));
  if (!ids || !c) {
    free(ids);
    free(c);
    return 0;
  }
  memcpy(ids, cand, m * sizeof(uint32_t));
  qsort(ids, m, sizeof(uint32_t), u32_cmp);
  uint64_t u = 0;
  for (uint64_t i = 0; i < m; ++i) {
    if (ids[i] == VO_NONE || ids[i] == p_id) continue;
    if (i > 0 && ids[i] == ids[i - 1]) continue;
    c[u].id = ids[i];
    c[u].dist = vo_distance(p_vec, row_ptr(D, ids[i]), D->d, D->dtype, D->metric);
    c[u].done = 0;
    ++u;
  }
  qsort(c, u, sizeof(cand_t), cand_cmp);

  uint32_t nout = 0;
  uint64_t pair = 0;
  for (uint64_t i = 0; i < u; ++i) {
    if (c[i].done) continue;
    /* p* = closest remaining candidate */
    out[nout++] = c[i].id;
    if (nout == R) break;
    const void* star = row_ptr(D, c[i].id);
    for (uint64_t j = i + 1; j < u; ++j) {
      if (c[j].done) continue;
      double dsc = vo_distance(star, row_ptr(D, c[j].id), D->d, D->dtype, D->metric);
      ++pair;
      if (alpha_dominates(D->dtype, alpha, dsc, c[j].dist)) c[j].done = 1;
    }
  }
  if (stats) {
    stats->prune_cand += u;
    stats->prune_evals += pair;
  }
  free(ids);
  free(c);
  return nout;
}

/* ------------------------------------------------------------------ */
/* start vertex, insertion order, schedule                              */
/* ------------------------------------------------------------------ */

uint32_t vo_start_vertex(const vo_data* D) {
  uint64_t n = D->n;
  uint32_t d = D->d;
  if (D->dtype == VO_U8 || D->dtype == VO_I8) {
    /* argmin ||x - S/n||^2  ==  argmin  n*||x||^2 - 2<x,S>   (exact, int64) */
    int64_t* S = (int64_t*)calloc(d, sizeof(int64_t));
    for (uint64_t i = 0; i < n; ++i)
      for (uint32_t j = 0; j < d; ++j)
        S[j] += D->dtype == VO_U8 ? (int64_t)((const uint8_t*)row_ptr(D, i))[j]
                                  : (int64_t)((const int8_t*)row_ptr(D, i))[j];
    uint32_t best = 0;
    int64_t best_score = 0;
    for (uint64_t i = 0; i < n; ++i) {
      int64_t nn = 0, xs = 0;
      for (uint32_t j = 0; j < d; ++j) {
        int64_t x = D->dtype == VO_U8 ? (int64_t)((const uint8_t*)row_ptr(D, i))[j]
                                      : (int64_t)((const int8_t*)row_ptr(D, i))[j];
        nn += x * x;
        xs += x * S[j];
      }
      int64_t score = (int64_t)n * nn - 2 * xs;
      if (i == 0 || score < best_score) {
        best = (uint32_t)i;
        best_score = score;
      }
    }
    free(S);
    return best;
  }
  double* mean = (double*)calloc(d, sizeof(double));
  for (uint64_t i = 0; i < n; ++i)
    for (uint32_t j = 0; j < d; ++j) mean[j] += ((const float*)row_ptr(D, i))[j];
  for (uint32_t j = 0; j < d; ++j) mean[j] /= (double)n;
  uint32_t best = 0;
  double best_score = 0;
  for (uint64_t i = 0; i < n; ++i) {
    double s = 0;
    for (uint32_t j = 0; j < d; ++j) {
      double t = ((const float*)row_ptr(D, i))[j] - mean[j];
      s += t * t;
    }
    if (i == 0 || s < best_score) {
      best = (uint32_t)i;
      best_score = s;
    }
  }
  free(mean);
  return best;
}

static uint64_t splitmix64(uint64_t* state) {
  uint64_t z = (*state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

/* Fisher-Yates from the front: step i = 0, 1, ..., m-2 draws the next output r
 * of SplitMix64(seed) and exchanges positions i and i + floor(r * (m - i) / 2^64),
 * a uniform choice among the positions not yet fixed.  Position i is final once
 * step i is done, so the order can be consumed while it is still being drawn.  */
static void shuffle_from_the_front(uint32_t* order, uint64_t m, uint64_t seed) {
  uint64_t state = seed;
  for (uint64_t i = 0; i + 1 < m; ++i) {
    uint64_t r = splitmix64(&state);
    uint64_t j = i + (uint64_t)(((unsigned __int128)r * (unsigned __int128)(m - i)) >> 64);
    uint32_t t = order[i];
    order[i] = order[j];
    order[j] = t;
  }
}

void vo_insertion_order(uint64_t n, uint32_t start, uint64_t seed, uint32_t* order) {
  uint64_t m = 0;
  for (uint64_t i = 0; i < n; ++i)
    if (i != start) order[m++] = (uint32_t)i;
  shuffle_from_the_front(order, m, seed);
}

uint64_t vo_schedule(uint64_t m, uint64_t theta, uint64_t* bounds) {
  if (theta < 1) theta = 1;
  uint64_t done = 0, rounds = 0;
  if (bounds) bounds[0] = 0;
  while (done < m) {
    /* Alg. 3 with 1-based start = done+1 over the ordered points: the batch
     * start..min(2*start, ...) has start+1 points; capped by theta and by
     * what is left.                                                        */
    uint64_t size = done + 2;
    if (size > theta) size = theta;
    if (size > m - done) size = m - done;
    done += size;
    ++rounds;
    if (bounds) bounds[rounds] = done;
  }
  return rounds;
}

/* ------------------------------------------------------------------ */
/* Alg. 2: insert(p, s, R, L)                                           */
/* ------------------------------------------------------------------ */

static uint32_t row_degree(const uint32_t* row, uint32_t R) {
  uint32_t deg = 0;
  while (deg < R && row[deg] != VO_NONE) ++deg;
  return deg;
}

int vo_insert(const vo_data* D, uint32_t* graph, uint32_t R, uint32_t start, uint32_t p,
              uint32_t L, double alpha, vo_stats* stats) {
  work_t w;
  if (work_init(&w, D->n, L, R)) {
    work_free(&w);
    return -1;
  }
  vo_stats st;
  memset(&st, 0, sizeof(st));
  uint64_t nv = 0, nb = 0;
  int rc = greedy_core(D, graph, R, start, row_ptr(D, p), L, 1, -1.0, &w, &nv, &nb, &st);
  if (rc) {
    work_free(&w);
    return rc;
  }
  uint32_t* ids = (uint32_t*)malloc((nv + R + 1) * sizeof(uint32_t));
  for (uint64_t i = 0; i < nv; ++i) ids[i] = w.vis[i].id;
  uint32_t* prow = graph + (size_t)p * R;
  vo_prune(D, row_ptr(D, p), p, ids, nv, R, alpha, prow, &st);
  st.prunes += 1;
  uint32_t pdeg = row_degree(prow, R);
  for (uint32_t j = 0; j < pdeg; ++j) {
    uint32_t q = prow[j];
    uint32_t* qrow = graph + (size_t)q * R;
    uint32_t qdeg = row_degree(qrow, R);
    st.edges += 1;
    if (qdeg < R) {
      qrow[qdeg] = p;
      st.appends += 1;
    } else {
      memcpy(ids, qrow, qdeg * sizeof(uint32_t));
      ids[qdeg] = p;
      vo_prune(D, row_ptr(D, q), q, ids, qdeg + 1, R, alpha, qrow, &st);
      st.reprunes += 1;
    }
  }
  free(ids);
  work_free(&w);
  stats_add(stats, &st);
  return 0;
}

int vo_build_sequential(const vo_data* D, uint32_t R, uint32_t L, double alpha, uint32_t start,
                        const uint32_t* order, uint64_t m, uint32_t* graph, vo_stats* stats) {
  memset(graph, 0xFF, (size_t)D->n * R * sizeof(uint32_t));
  for (uint64_t i = 0; i < m; ++i) {
    int rc = vo_insert(D, graph, R, start, order[i], L, alpha, stats);
    if (rc) return rc;
  }
  return 0;
}

/* ------------------------------------------------------------------ */
/* Alg. 3: BatchInsert and batchBuild                                   */
/* ------------------------------------------------------------------ */

typedef struct {
  uint32_t dst; /* existing point b          */
  uint32_t src; /* batch point p             */
  uint64_t seq; /* position in emission order */
} edge_t;

static int edge_cmp(const void* pa, const void* pb) {
  const edge_t* a = (const edge_t*)pa;
  const edge_t* b = (const edge_t*)pb;
  if (a->dst != b->dst) return a->dst < b->dst ? -1 : 1;
  if (a->seq != b->seq) return a->seq < b->seq ? -1 : 1;
  return 0;
}

int vo_batch_insert(const vo_data* D, uint32_t* graph, uint32_t R, uint32_t start,
                    const uint32_t* batch, uint64_t b, uint32_t L, double alpha, int threads,
                    vo_stats* stats) {
  return vo_batch_insert_from(D, graph, R, start, NULL, batch, b, L, alpha, threads, NULL, stats);
}

int vo_batch_insert_from(const vo_data* D, uint32_t* graph, uint32_t R, uint32_t start,
                         const uint32_t* starts, const uint32_t* batch, uint64_t b, uint32_t L,
                         double alpha, int threads, uint32_t* nearest_out, vo_stats* stats) {
  if (b == 0) return 0;
  int nthreads = vo_threads(threads);
  (void)nthreads;
  uint32_t* newrows = (uint32_t*)malloc((size_t)b * R * sizeof(uint32_t));
  if (!newrows) return -1;
  int err = 0;

  /* step 1: every batch point searches the graph as it stood before this
   * batch and prunes its visited set; the rows are held back until the
   * loop is over, so the graph really is immutable meanwhile.             */
#pragma omp parallel num_threads(nthreads)
  {
    work_t w;
    int bad = work_init(&w, D->n, L, R);
    vo_stats st;
    memset(&st, 0, sizeof(st));
    uint32_t* ids = NULL;
    uint64_t ids_cap = 0;
#pragma omp for schedule(dynamic, 16)
    for (int64_t i = 0; i < (int64_t)b; ++i) {
      if (bad) continue;
      uint32_t p = batch[i];
      uint64_t nv = 0, nb = 0;
      int rc = greedy_core(D, graph, R, starts ? starts[i] : start, row_ptr(D, p), L, 1, -1.0, &w,
                           &nv, &nb, &st);
      if (rc) {
        bad = rc;
        continue;
      }
      if (nearest_out) nearest_out[i] = w.beam[0].id; /* the closest vertex of V */
      if (nv > ids_cap) {
        ids_cap = nv * 2;
        ids = (uint32_t*)realloc(ids, ids_cap * sizeof(uint32_t));
      }
      for (uint64_t j = 0; j < nv; ++j) ids[j] = w.vis[j].id;
      vo_prune(D, row_ptr(D, p), p, ids, nv, R, alpha, newrows + (size_t)i * R, &st);
      st.prunes += 1;
    }
#pragma omp critical
    {
      stats_add(stats, &st);
      if (bad) err = bad;
    }
    free(ids);
    work_free(&w);
  }
  if (err) {
    free(newrows);
    return err;
  }
  for (uint64_t i = 0; i < b; ++i)
    memcpy(graph + (size_t)batch[i] * R, newrows + (size_t)i * R, R * sizeof(uint32_t));

  /* step 2: collect (u = batch point, v = existing point), bring equal v
   * together (a sort stands in for the semisort), add, prune on overflow.  */
  uint64_t ne = 0;
  for (uint64_t i = 0; i < b; ++i) ne += row_degree(newrows + (size_t)i * R, R);
  edge_t* E = (edge_t*)malloc((ne ? ne : 1) * sizeof(edge_t));
  uint64_t* seg = (uint64_t*)malloc((ne + 1) * sizeof(uint64_t));
  if (!E || !seg) {
    free(newrows);
    free(E);
    free(seg);
    return -1;
  }
  uint64_t e = 0;
  for (uint64_t i = 0; i < b; ++i) {
    const uint32_t* row = newrows + (size_t)i * R;
    uint32_t deg = row_degree(row, R);
    for (uint32_t j = 0; j < deg; ++j) {
      E[e].dst = row[j];
      E[e].src = batch[i];
      E[e].seq = e;
      ++e;
    }
  }
  qsort(E, ne, sizeof(edge_t), edge_cmp);
  uint64_t nseg = 0;
  for (uint64_t i = 0; i < ne; ++i)
    if (i == 0 || E[i].dst != E[i - 1].dst) seg[nseg++] = i;
  seg[nseg] = ne;

#pragma omp parallel num_threads(nthreads)
  {
    vo_stats st;
    memset(&st, 0, sizeof(st));
    uint32_t* U = NULL;
    uint64_t U_cap = 0;
    int bad = 0;
#pragma omp for schedule(dynamic, 64)
    for (int64_t s = 0; s < (int64_t)nseg; ++s) {
      uint64_t lo = seg[s], hi = seg[s + 1];
      uint32_t dst = E[lo].dst;
      uint32_t* drow = graph + (size_t)dst * R;
      uint32_t deg = row_degree(drow, R);
      uint64_t cnt = hi - lo;
      if (deg + cnt > U_cap) {
        U_cap = (deg + cnt) * 2;
        U = (uint32_t*)realloc(U, U_cap * sizeof(uint32_t));
      }
      memcpy(U, drow, deg * sizeof(uint32_t));
      for (uint64_t j = 0; j < cnt; ++j) {
        uint32_t src = E[lo + j].src;
        /* sources are new this round, so never present already, and a
         * destination is never a point of this batch                       */
        for (uint32_t t = 0; t < deg; ++t)
          if (drow[t] == src) bad = -3;
        U[deg + j] = src;
      }
      st.edges += cnt;
      if (deg + cnt <= R) {
        memcpy(drow, U, (deg + cnt) * sizeof(uint32_t));
        st.appends += 1;
      } else {
        vo_prune(D, row_ptr(D, dst), dst, U, deg + cnt, R, alpha, drow, &st);
        st.reprunes += 1;
      }
    }
#pragma omp critical
    {
      stats_add(stats, &st);
      if (bad) err = bad;
    }
    free(U);
  }
  free(newrows);
  free(E);
  free(seg);
  return err;
}

int vo_build(const vo_data* D, uint32_t R, uint32_t L, double alpha, uint64_t seed,
             uint64_t theta, uint32_t start, const uint32_t* order, uint64_t max_rounds,
             int threads, uint32_t* graph, uint32_t* start_out, vo_stats* stats) {
  if (!D || !graph || D->n < 1 || R < 1 || L < 1) return -1;
  uint64_t n = D->n, m = n - 1;
  if (start == VO_NONE) start = vo_start_vertex(D);
  if (start >= n) return -1;
  if (start_out) *start_out = start;
  if (theta == 0) theta = n / 50 > 1 ? n / 50 : 1;
  uint32_t* own = NULL;
  if (!order) {
    own = (uint32_t*)malloc((m ? m : 1) * sizeof(uint32_t));
    if (!own) return -1;
    vo_insertion_order(n, start, seed, own);
    order = own;
  }
  memset(graph, 0xFF, (size_t)n * R * sizeof(uint32_t));
  uint64_t rounds = vo_schedule(m, theta, NULL);
  uint64_t* bounds = (uint64_t*)malloc((rounds + 1) * sizeof(uint64_t));
  vo_schedule(m, theta, bounds);
  int rc = 0;
  for (uint64_t r = 0; r < rounds; ++r) {
    if (max_rounds && r >= max_rounds) break;
    rc = vo_batch_insert(D, graph, R, start, order + bounds[r], bounds[r + 1] - bounds[r], L,
                         alpha, threads, stats);
    if (stats) stats->rounds += 1;
    if (rc) break;
  }
  free(bounds);
  free(own);
  return rc;
}

/* ------------------------------------------------------------------ */
/* streaming insertion of new points: BatchInsert of Alg. 3 applied to   */
/* points that arrive after the build, the schedule of Sec. 3.1 carried  */
/* on from the points already present                                    */
/* ------------------------------------------------------------------ */

void vo_new_points_order(uint64_t first, uint64_t count, uint64_t seed, uint32_t* order) {
  for (uint64_t i = 0; i < count; ++i) order[i] = (uint32_t)(first + i);
  shuffle_from_the_front(order, count, seed);
}

uint64_t vo_schedule_from(uint64_t present, uint64_t m, uint64_t theta, uint64_t* bounds) {
  if (theta < 1) theta = 1;
  uint64_t taken = 0, rounds = 0;
  if (bounds) bounds[0] = 0;
  while (taken < m) {
    /* a batch may at most double what is there (present + taken points
     * besides the start vertex, plus the start vertex itself, plus one, as
     * in the build), is capped by theta and by what is left                */
    uint64_t size = present + taken + 2;
    if (size > theta) size = theta;
    if (size > m - taken) size = m - taken;
    taken += size;
    ++rounds;
    if (bounds) bounds[rounds] = taken;
  }
  return rounds;
}

int vo_insert_points(const vo_data* D, uint32_t* graph, uint32_t R, uint32_t start, uint64_t n_old,
                     uint32_t L, double alpha, uint64_t seed, uint64_t theta,
                     const uint32_t* order, uint64_t max_rounds, int threads, vo_stats* stats) {
  if (!D || !graph || R < 1 || L < 1 || n_old < 1 || n_old > D->n || start >= n_old) return -1;
  uint64_t n = D->n, m = n - n_old;
  if (m == 0) return 0;
  if (theta == 0) theta = n / 50 > 1 ? n / 50 : 1;
  uint32_t* own = NULL;
  if (!order) {
    own = (uint32_t*)malloc(m * sizeof(uint32_t));
    if (!own) return -1;
    vo_new_points_order(n_old, m, seed, own);
    order = own;
  } else {
    /* every new id exactly once */
    unsigned char* seen = (unsigned char*)calloc(m, 1);
    if (!seen) return -1;
    int bad = 0;
    for (uint64_t i = 0; i < m && !bad; ++i) {
      if (order[i] < n_old || order[i] >= n || seen[order[i] - n_old]) bad = 1;
      else seen[order[i] - n_old] = 1;
    }
    free(seen);
    if (bad) return -1;
  }
  uint64_t rounds = vo_schedule_from(n_old - 1, m, theta, NULL);
  uint64_t* bounds = (uint64_t*)malloc((rounds + 1) * sizeof(uint64_t));
  if (!bounds) {
    free(own);
    return -1;
  }
  vo_schedule_from(n_old - 1, m, theta, bounds);
  int rc = 0;
  for (uint64_t r = 0; r < rounds; ++r) {
    if (max_rounds && r >= max_rounds) break;
    rc = vo_batch_insert(D, graph, R, start, order + bounds[r], bounds[r + 1] - bounds[r], L,
                         alpha, threads, stats);
    if (stats) stats->rounds += 1;
    if (rc) break;
  }
  free(bounds);
  free(own);
  return rc;
}

/* ------------------------------------------------------------------ */
/* batched queries and exhaustive search                                */
/* ------------------------------------------------------------------ */

static void store_dist(void* out, uint64_t idx, int dtype, double dist, int valid) {
  if (dtype == VO_F32)
    ((float*)out)[idx] = valid ? (float)dist : INFINITY;
  else
    ((int32_t*)out)[idx] = valid ? (int32_t)dist : INT32_MAX;
}

int vo_search_batch(const vo_data* D, const uint32_t* graph, uint32_t R, uint32_t start,
                    const void* queries, uint64_t nq, uint32_t k, uint32_t L, int threads,
                    uint32_t* ids_out, void* dists_out, vo_stats* stats) {
  return vo_search_batch_eps(D, graph, R, start, queries, nq, k, L, -1.0, threads, ids_out, dists_out, stats);
}

int vo_search_batch_eps(const vo_data* D, const uint32_t* graph, uint32_t R, uint32_t start,
                        const void* queries, uint64_t nq, uint32_t k, uint32_t L, double eps,
                        int threads, uint32_t* ids_out, void* dists_out, vo_stats* stats) {
  return vo_search_batch_from(D, graph, R, start, NULL, queries, nq, k, L, eps, threads, ids_out,
                              dists_out, stats);
}

int vo_search_batch_from(const vo_data* D, const uint32_t* graph, uint32_t R, uint32_t start,
                         const uint32_t* starts, const void* queries, uint64_t nq, uint32_t k,
                         uint32_t L, double eps, int threads, uint32_t* ids_out, void* dists_out,
                         vo_stats* stats) {
  if (!D || !graph || !queries || k < 1 || k > L) return -1;
  if (!starts && start >= D->n) return -1;
  if (starts)
    for (uint64_t q = 0; q < nq; ++q)
      if (starts[q] >= D->n) return -1;
  if (!(eps < 16384.0)) return -1;
  int nthreads = vo_threads(threads);
  (void)nthreads;
  int err = 0;
  size_t qbytes = (size_t)D->d * elem_size(D->dtype);
#pragma omp parallel num_threads(nthreads)
  {
    work_t w;
    int bad = work_init(&w, D->n, L, R);
    vo_stats st;
    memset(&st, 0, sizeof(st));
#pragma omp for schedule(dynamic, 16)
    for (int64_t q = 0; q < (int64_t)nq; ++q) {
      if (bad) continue;
      uint64_t nv = 0, nb = 0;
      int rc = greedy_core(D, graph, R, starts ? starts[q] : start,
                           (const char*)queries + (size_t)q * qbytes, L, k, eps, &w, &nv, &nb, &st);
      if (rc) {
        bad = rc;
        continue;
      }
      for (uint32_t i = 0; i < k; ++i) {
        int valid = i < nb;
        ids_out[(size_t)q * k + i] = valid ? w.beam[i].id : VO_NONE;
        if (dists_out)
          store_dist(dists_out, (size_t)q * k + i, D->dtype, valid ? w.beam[i].dist : 0.0, valid);
      }
    }
#pragma omp critical
    {
      stats_add(stats, &st);
      if (bad) err = bad;
    }
    work_free(&w);
  }
  return err;
}

int vo_brute_force(const vo_data* D, const void* queries, uint64_t nq, uint32_t k, int threads,
                   uint32_t* ids_out, void* dists_out) {
  if (!D || !queries || k < 1) return -1;
  int nthreads = vo_threads(threads);
  (void)nthreads;
  size_t qbytes = (size_t)D->d * elem_size(D->dtype);
#pragma omp parallel num_threads(nthreads)
  {
    cand_t* top = (cand_t*)malloc(((size_t)k + 1) * sizeof(cand_t));
#pragma omp for schedule(dynamic, 4)
    for (int64_t q = 0; q < (int64_t)nq; ++q) {
      const void* qv = (const char*)queries + (size_t)q * qbytes;
      uint32_t cnt = 0;
      for (uint64_t i = 0; i < D->n; ++i) {
        cand_t c;
        c.dist = vo_distance(qv, row_ptr(D, i), D->d, D->dtype, D->metric);
        c.id = (uint32_t)i;
        c.done = 0;
        if (cnt == k && !cand_less(&c, &top[k - 1])) continue;
        uint32_t pos = cnt < k ? cnt : k - 1;
        while (pos > 0 && cand_less(&c, &top[pos - 1])) {
          top[pos] = top[pos - 1];
          --pos;
        }
        top[pos] = c;
        if (cnt < k) ++cnt;
      }
      for (uint32_t i = 0; i < k; ++i) {
        int valid = i < cnt;
        ids_out[(size_t)q * k + i] = valid ? top[i].id : VO_NONE;
        store_dist(dists_out, (size_t)q * k + i, D->dtype, valid ? top[i].dist : 0.0, valid);
      }
    }
    free(top);
  }
  return 0;
}
