// Host-visible declarations shared by the translation units of the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace annmi {

using u32 = uint32_t;
using u64 = uint64_t;

// Which template instance serves a (dtype, metric, d) combination.
struct DistCfg {
  int kind;       // Kind
  int vec;        // bytes per load: 16 or 4
  int nch;        // pieces per lane: 1, 2, 4 or 8
  u32 npieces;    // pieces per row
  u64 row_bytes;  // d * sizeof(element)
};

// Device-side counters (all commutative integer sums).  Thousands of wavefronts adding to one
// address queue up at a single memory channel and slow every other access that goes there, so
// there are COUNTER_COPIES copies, each on a cache line of its own; a block adds to the copy
// picked by its index and the host adds the copies up.
struct alignas(128) DevCounters {
  unsigned long long searches, hops, evals, prunes, reprunes, appends, edges, prune_evals;
  unsigned long long passes, survivors, insert_hops;  // search kernel: 8-vertex distance passes, beam insertions, hops with an insertion
};
constexpr u32 COUNTER_COPIES = 1024;
__device__ __forceinline__ DevCounters* block_counters(DevCounters* base) {
  return base + (blockIdx.x & (COUNTER_COPIES - 1u));
}

struct SearchArgs {
  const char* points;     // vectors of the graph's vertices
  const u32* graph;       // n x R
  const char* queries;    // query vectors (the points themselves during a build)
  const u32* qidx;        // optional: query i is row qidx[i] of `queries`
  u64 qrow_bytes;
  u32 nq;
  u32 R;
  u32 start;
  // Layered index (Sec. 4.2): a start vertex of its own for every search.  Search i works on
  // position p = slot ? slot[i] : i of two arrays: it starts at starts[p] (when `starts` is
  // given, else at `start`) and leaves the closest vertex it found, passed through `down` when
  // that is given (the vertex's id one layer below), in next_start[p] (when given).  starts and
  // next_start may be the same array: a search touches its own position only.
  const u32* starts;
  const u32* slot;
  const u32* down;
  u32* next_start;
  u32 L;
  u32 k;
  u32* batch_counters;  // build only: the batch's counter words (overflow count [0], arena top [4..5], work
                        // list lengths [8..11]); workgroup 0 zeroes them for the steps that follow
  // (1 + eps) rule of the search (Sec. 4.5): off when eps16 < 0; integer kinds use eps16 =
  // round(eps * 2^16), float kinds epsf
  long long eps16;
  float epsf;
  u32 hash_buckets;  // 16-byte buckets of the visited filter (any count from 4 to 2048)
  u32 id_bits;       // > 0: the filter stores tags of ids that fit in this many bits ...
  u32 tag_width;     // ... eight of 16 bits or six of 21 bits per bucket (0: four 32-bit ids)
  // build: visited list, one slot of vis_cap keys per search (may be null).  A search that
  // outgrows its slot moves its list to a chunk of vis_cap + spill_chunk keys taken from `spill`
  // (if given) and records the chunk's offset in vis_where[search] (~0 = still in its slot).
  u64* vis;
  u32* nvis;
  u32 vis_cap;
  u64* spill;
  u64 spill_cap;
  unsigned long long* spill_top;
  u32 spill_chunk;
  u64* vis_where;
  // query: results (out_ids may be null: then nothing is written; out_dists may be null)
  u32* out_ids;
  void* out_dists;
  DevCounters* counters;  // may be null
};

// The walk of a query through the upper layers of the layered index (Sec. 4.2): a search with
// beam 1 per layer, from the top down.
struct DescendLayer {
  const char* points;  // the layer's vectors
  const u32* graph;    // its adjacency rows, R ids each
  const u32* down;     // id of each of its vertices one layer below
  u32 R;
  u32 pad_;
};
struct DescendArgs {
  const char* queries;
  u64 qrow_bytes;
  u32 nq;
  u32 nlayers;                 // layers walked, listed from the top
  u32 entry;                   // the entry point's id on the first of them
  const DescendLayer* layers;  // device
  u32* out;                    // nq ids on the layer below the last one walked
};

struct PruneArgs {
  const char* points;
  u32* graph;  // rows of the batch points are written
  const u32* qidx;      // batch point ids
  const u32* slotmap;   // optional: search i belongs to batch slot slotmap[i]
  u32 nq;
  u32 R;
  const u64* vis;
  const u32* nvis;
  u32 vis_cap;
  u64* vis_rw;          // same memory as vis: lists longer than the LDS buffer are pruned in place
  u64* spill;           // chunks of vis_cap + spill_chunk keys for lists that outgrew their slot
  u32 spill_chunk;
  const u64* vis_where; // per search: offset of its chunk in spill, or ~0 (may be null)
  unsigned long long* spill_top_reset;  // optional: zeroed by workgroup 0 for the next batch's searches
  u32* lost_flag;       // set (and left set) when a list did not fit anywhere
  u32* meta;            // per row: degree | clean prefix length << 16 (written for the batch points)
  u64* edges;           // batch_size x R keys (dest << 32 | source), ~0 in unused slots
  u32 stage_bytes;      // dynamic LDS for the selected points' vectors (0: read them from memory)
  u32 use_mfma;         // u8/i8 rows up to 128 B: pair distances on the matrix cores
  u32* overflow_count;  // searches whose visited list did not fit
  u32* overflow_list;   // their indices
  long long a16;
  float af;
  DevCounters* counters;
};

// One overflowing row of step 2: its segment of the sorted edge keys and what the planning pass
// already knows about the row, so that the worker need not chase keys[i0] -> meta[b] first.
struct alignas(16) MergeItem {
  u32 i0;    // index of the segment's first key
  u32 cnt;   // segment length
  u32 b;     // the row
  u32 meta;  // its degree and clean-prefix length before this round's edges
};

struct MergeArgs {
  const char* points;
  u32* graph;
  u32* meta;  // per row: degree | clean prefix length << 16
  u32 R;
  const u64* keys;  // sorted edge keys (dest << 32 | source)
  u64 nkeys;
  u32* list_count;     // [4]: segments filed for the fast / gram / large / medium re-prune
  // the four work lists; the medium list shares the large one's array and grows down from its
  // last element (item k at list_items[3][-k]): a segment is in one of the two
  MergeItem* list_items[4];
  u32 medium_max;      // candidate lists of up to this length go to the medium list (0: no such list)
  u32 fast_amax;       // most new entries the fast path takes
  u32 gram_ok;         // the matrix-core path applies to this dtype / row size
  u32 gram_tmax;       // and to at most this many candidates
  u32 stage_bytes;     // dynamic LDS of the generic kernel for the selected points' vectors
  u32 use_mfma;        // the generic kernel takes pair distances on the matrix cores
  u64* arena;          // spill space for candidate lists that do not fit in LDS
  u64 arena_cap;
  unsigned long long* arena_top;
  u32* error_flag;
  long long a16;
  float af;
  DevCounters* counters;
  u32 force_prune;  // non-zero: every segment is pruned, also where row and segment fit in R (the
                    // clustering-based builder, Sec. 4.3; rows start empty there)
};

constexpr u32 PRUNE_LDS_CAP = 512;     // candidate keys sorted in LDS by the step-1 prune kernel (a power of two)
constexpr u32 MERGE_MEDIUM_MAX = 512;  // step-2 candidate lists up to this length have a kernel instance of their own
constexpr u32 MERGE_SPILL_MIN = 4096;  // step-2 candidate lists longer than this go to the spill arena (a power of two)
constexpr u32 STAGE_BUDGET = 10240;    // LDS bytes the prune kernels may spend on the selected points' vectors

// launchers (each returns the hipGetLastError() of its launches)
hipError_t launch_search(const DistCfg& cfg, const SearchArgs& a, hipStream_t s);
hipError_t launch_descend(const DistCfg& cfg, const DescendArgs& a, hipStream_t s);
hipError_t launch_prune(const DistCfg& cfg, const PruneArgs& a, hipStream_t s);
hipError_t launch_plan(const MergeArgs& a, hipStream_t s);
hipError_t launch_merge(const DistCfg& cfg, const MergeArgs& a, u32 grid, hipStream_t s, hipStream_t s_gram,
                        hipStream_t s_generic, hipStream_t s_medium);
hipError_t launch_meta_from_rows(const u32* graph, u64 n, u32 R, u32* meta, hipStream_t s);
hipError_t launch_meta_forget_clean(u64 n, u32* meta, hipStream_t s);
bool gram_path_ok(const DistCfg& cfg);
u32 gram_path_tmax();
u32 fast_path_amax(const DistCfg& cfg);
u32 prune_stage_bytes(u32 R, const DistCfg& cfg);
bool mfma_prune_ok(u32 R, const DistCfg& cfg);

// stable LSD radix sort of 64-bit keys on bits [32, 32+key_bits); result is left in `keys`
// (`tmp` holds `count` keys, `hist` holds radix_hist_entries(count) u32)
u64 radix_hist_entries(u64 count);
hipError_t radix_sort_edges(u64* keys, u64* tmp, u32* hist, u64 hist_entries, u64 count, u32 key_bits, hipStream_t s,
                            u32 first_bit = 32);

// start vertex (point nearest the mean)
hipError_t start_vertex_device(const void* points, u64 n, u32 d, int dtype, hipStream_t s, u32* start_out);

u32 search_lds_bytes(u32 L, u32 hash_buckets);
u32 search_hash_buckets(u32 L, u32 hash_bits);  // hash_bits: the caller's explicit choice, or 0
// how the visited filter stores vertices of a graph of n points: fills id_bits and tag_width
void search_filter_mode(u64 n, u32 hash_buckets, u32* id_bits, u32* tag_width);

}  // namespace annmi
