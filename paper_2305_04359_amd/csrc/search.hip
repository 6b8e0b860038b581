// Host side of the beam search: sizes of the per-wave LDS, the filter layout, and the launch of
// the kernel variants without the (1 + eps) rule (the graph build and plain queries).  The
// variants with the rule, and those of the layered index, are compiled in translation units of
// their own, in parallel.
#include "ann_dispatch.hpp"
#include "search_kernel.hpp"

namespace annmi {

u32 search_lds_bytes(u32 L, u32 hash_buckets) { return search_nslot_for(L) * 64 * 8 + 64 * 8 + hash_buckets * 16; }

// Size of the visited filter.  An explicit hash_bits (log2 of the size in 32-bit words) is taken
// as it is.  Otherwise: 8 words per beam entry, rounded up to a power of two, but never more than
// 1,024 words (512 for beams above 512 entries), then adjusted so that the wave's LDS lands
// exactly on the next occupancy step (waves per CU a multiple of four, at most 32, LDS handed
// out in 512-byte units of 160 KB).  Occupancy is worth more than the evaluations a larger table
// saves: measured on 128-d uint8 data at beam 128 (a million points), and at beams of 200 to
// 2,048 on a hundred million points, where tables of 1,024 and 512 words answer 1.7 to 2.3 times
// the queries per second of tables of 4,096 and 8,192.  The table is never cut below 3/4 of the
// power of two.
u32 search_hash_buckets(u32 L, u32 hash_bits) {
  if (hash_bits) return 1u << (hash_bits - 2u);
  u32 want = 8u * L, bits = 9;
  while ((1u << bits) < want && bits < (L > 512u ? 9u : 10u)) ++bits;
  const u32 full = 1u << (bits - 2u);
  const u32 base = search_lds_bytes(L, 0);
  const u32 lds_full = (search_lds_bytes(L, full) + 511u) & ~511u;
  u32 waves = 163840u / lds_full;
  waves = (waves + 3u) & ~3u;
  if (waves > 32u) waves = 32u;
  const u32 budget = (163840u / waves) & ~511u;
  if (budget <= base) return full;
  u32 nb = (budget - base) / 16u;
  if (nb < full - full / 4u) return full;
  if (nb > full) nb = full;
  return nb;
}

// Tags identify a vertex exactly when ids fit id_bits bits and the tag keeps the id_bits -
// floor(log2 buckets) low bits of the mixed id: 16-bit tags carry up to 15 of them (0xFFFF marks
// an empty slot), 21-bit tags up to 20.
void search_filter_mode(u64 n, u32 hash_buckets, u32* id_bits, u32* tag_width) {
  u32 bits = 1;
  while ((1ull << bits) < n) ++bits;  // ids < n <= 2^bits
  u32 q = 0;
  while ((2u << q) <= hash_buckets) ++q;  // floor(log2(buckets))
  if (bits < q + 1u) bits = q + 1u;
  *id_bits = 0;
  *tag_width = 0;
  if (bits <= 24u && bits - q <= 15u) {
    *id_bits = bits;
    *tag_width = 16;
  } else if (bits <= 31u && bits - q <= 20u) {
    *id_bits = bits;
    *tag_width = 21;
  }
}

template <int KIND, int VEC, int NCH>
static hipError_t launch_plain(const SearchArgs& a, const VecTable& T, hipStream_t s) {
  return launch_search_variant<KIND, VEC, NCH, false, false>(a, T, s);
}

static hipError_t launch_search_plain(const DistCfg& cfg, const SearchArgs& a, const VecTable& T, hipStream_t s) {
  ANN_DISPATCH_CFG(launch_plain, a, T, s);
}

hipError_t launch_search(const DistCfg& cfg, const SearchArgs& a, hipStream_t s) {
  if (a.nq == 0) return hipSuccess;
  VecTable T{a.points, (u32)cfg.row_bytes, cfg.npieces};
  const bool own = a.starts != nullptr || a.next_start != nullptr;
  if (own) return a.eps16 >= 0 ? launch_search_own_eps(cfg, a, T, s) : launch_search_own(cfg, a, T, s);
  return a.eps16 >= 0 ? launch_search_eps(cfg, a, T, s) : launch_search_plain(cfg, a, T, s);
}

}  // namespace annmi
