/*
 * hnsw_oracle.c -- TEST INFRASTRUCTURE, not product code.  See hnsw_oracle.h.
 */
#include "hnsw_oracle.h"

#include <stdlib.h>
#include <string.h>

static size_t elem_bytes(int dtype) { return dtype == VO_F32 ? 4 : 1; }

static uint32_t layer_degree(const vo_hnsw* h, uint32_t l) { return l ? h->m : 2 * h->m; }

uint32_t vo_hnsw_level(uint64_t seed, uint32_t id, uint32_t m) {
  /* the (id+1)-th output of SplitMix64(seed) */
  uint64_t z = seed + ((uint64_t)id + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  uint64_t r = z ^ (z >> 31);
  uint32_t l = 0;
  uint64_t t = UINT64_MAX;
  if (m < 2) return 0;
  for (;;) {
    t /= m; /* floor((2^64 - 1) / m^(l+1)) */
    if (t == 0 || r > t) break;
    ++l;
  }
  return l;
}

void vo_hnsw_free(vo_hnsw* h) {
  if (!h) return;
  if (h->rows)
    for (uint32_t l = 0; l <= h->top; ++l) free(h->rows[l]);
  free(h->rows);
  free(h->level);
  free(h);
}

int vo_hnsw_insert_batch(const vo_data* D, vo_hnsw* h, const uint32_t* batch, uint64_t b,
                         uint32_t efc, double alpha, int threads, vo_stats* stats) {
  if (!D || !h || !batch || h->n != D->n) return -1;
  if (b == 0) return 0;
  size_t vbytes = (size_t)D->d * elem_bytes(D->dtype);
  uint32_t* cur = (uint32_t*)malloc(b * sizeof(uint32_t)); /* start vertex of every batch point */
  uint32_t* sel = (uint32_t*)malloc(b * sizeof(uint32_t)); /* positions in the batch           */
  uint32_t* ids = (uint32_t*)malloc(b * sizeof(uint32_t));
  uint32_t* sts = (uint32_t*)malloc(b * sizeof(uint32_t));
  uint32_t* got = (uint32_t*)malloc(b * sizeof(uint32_t));
  char* qbuf = (char*)malloc(b * vbytes);
  int rc = (cur && sel && ids && sts && got && qbuf) ? 0 : -1;
  if (rc == 0) {
    for (uint64_t i = 0; i < b; ++i) cur[i] = h->entry;
    for (uint32_t l = h->top;; --l) {
      uint32_t deg = layer_degree(h, l);
      /* points whose level is below l pass through: beam 1 over the layer as it is now, i.e.
       * as it stood before this batch (the batch's own insertion into it comes next) */
      uint64_t nd = 0;
      for (uint64_t i = 0; i < b; ++i)
        if (h->level[batch[i]] < l) {
          sel[nd] = (uint32_t)i;
          sts[nd] = cur[i];
          memcpy(qbuf + nd * vbytes, (const char*)D->points + (size_t)batch[i] * vbytes, vbytes);
          ++nd;
        }
      if (nd) {
        rc = vo_search_batch_from(D, h->rows[l], deg, 0, sts, qbuf, nd, 1, 1, -1.0, threads, got,
                                  NULL, stats);
        if (rc) break;
        for (uint64_t j = 0; j < nd; ++j) cur[sel[j]] = got[j];
      }
      /* points of this layer: BatchInsert from their own start vertices */
      uint64_t ni = 0;
      for (uint64_t i = 0; i < b; ++i)
        if (h->level[batch[i]] >= l) {
          sel[ni] = (uint32_t)i;
          sts[ni] = cur[i];
          ids[ni] = batch[i];
          ++ni;
        }
      if (ni) {
        rc = vo_batch_insert_from(D, h->rows[l], deg, 0, sts, ids, ni, efc, alpha, threads, got,
                                  stats);
        if (rc) break;
        for (uint64_t j = 0; j < ni; ++j) cur[sel[j]] = got[j];
      }
      if (l == 0) break;
    }
  }
  free(cur);
  free(sel);
  free(ids);
  free(sts);
  free(got);
  free(qbuf);
  return rc;
}

int vo_hnsw_build(const vo_data* D, uint32_t m, uint32_t efc, double alpha, uint64_t seed,
                  uint64_t theta, const uint32_t* level, const uint32_t* order,
                  uint64_t max_rounds, int threads, vo_hnsw** out, vo_stats* stats) {
  if (!D || !out || D->n < 1 || m < 2 || efc < 1) return -1;
  *out = NULL;
  uint64_t n = D->n;
  vo_hnsw* h = (vo_hnsw*)calloc(1, sizeof(vo_hnsw));
  if (!h) return -1;
  h->n = n;
  h->m = m;
  h->level = (uint32_t*)malloc(n * sizeof(uint32_t));
  if (!h->level) {
    vo_hnsw_free(h);
    return -1;
  }
  for (uint64_t i = 0; i < n; ++i) h->level[i] = level ? level[i] : vo_hnsw_level(seed, (uint32_t)i, m);
  /* entry point: highest level, smallest id */
  h->entry = 0;
  for (uint64_t i = 1; i < n; ++i)
    if (h->level[i] > h->level[h->entry]) h->entry = (uint32_t)i;
  h->top = h->level[h->entry];
  h->rows = (uint32_t**)calloc((size_t)h->top + 1, sizeof(uint32_t*));
  if (!h->rows) {
    vo_hnsw_free(h);
    return -1;
  }
  for (uint32_t l = 0; l <= h->top; ++l) {
    size_t bytes = (size_t)n * layer_degree(h, l) * sizeof(uint32_t);
    h->rows[l] = (uint32_t*)malloc(bytes);
    if (!h->rows[l]) {
      vo_hnsw_free(h);
      return -1;
    }
    memset(h->rows[l], 0xFF, bytes);
  }

  uint64_t cnt = n - 1;
  if (theta == 0) theta = n / 50 > 1 ? n / 50 : 1;
  uint32_t* own = NULL;
  if (!order) {
    own = (uint32_t*)malloc((cnt ? cnt : 1) * sizeof(uint32_t));
    if (!own) {
      vo_hnsw_free(h);
      return -1;
    }
    vo_insertion_order(n, h->entry, seed, own);
    order = own;
  }
  uint64_t rounds = vo_schedule(cnt, theta, NULL);
  uint64_t* bounds = (uint64_t*)malloc((rounds + 1) * sizeof(uint64_t));
  vo_schedule(cnt, theta, bounds);
  int rc = bounds ? 0 : -1;
  for (uint64_t r = 0; r < rounds && rc == 0; ++r) {
    if (max_rounds && r >= max_rounds) break;
    rc = vo_hnsw_insert_batch(D, h, order + bounds[r], bounds[r + 1] - bounds[r], efc, alpha, threads,
                              stats);
    if (stats) stats->rounds += 1;
  }
  free(bounds);
  free(own);
  if (rc) {
    vo_hnsw_free(h);
    return rc;
  }
  *out = h;
  return 0;
}

int vo_hnsw_search_batch(const vo_data* D, const vo_hnsw* h, const void* queries, uint64_t nq,
                         uint32_t k, uint32_t L, double eps, int threads, uint32_t* ids_out,
                         void* dists_out, uint32_t* entry_out, vo_stats* stats) {
  if (!D || !h || !queries || !ids_out || k < 1 || k > L || h->n != D->n) return -1;
  if (nq == 0) return 0;
  uint32_t* cur = (uint32_t*)malloc(nq * sizeof(uint32_t));
  uint32_t* got = (uint32_t*)malloc(nq * sizeof(uint32_t));
  if (!cur || !got) {
    free(cur);
    free(got);
    return -1;
  }
  for (uint64_t q = 0; q < nq; ++q) cur[q] = h->entry;
  int rc = 0;
  for (uint32_t l = h->top; l >= 1 && rc == 0; --l) {
    rc = vo_search_batch_from(D, h->rows[l], layer_degree(h, l), 0, cur, queries, nq, 1, 1, -1.0,
                              threads, got, NULL, stats);
    if (rc == 0) memcpy(cur, got, nq * sizeof(uint32_t));
  }
  if (rc == 0) {
    if (entry_out) memcpy(entry_out, cur, nq * sizeof(uint32_t));
    rc = vo_search_batch_from(D, h->rows[0], layer_degree(h, 0), 0, cur, queries, nq, k, L, eps,
                              threads, ids_out, dists_out, stats);
  }
  free(cur);
  free(got);
  return rc;
}
