// Arithmetic of the schedule that the host planner and the kernels must agree on, written once:
// which key tiles a work item walks.  Plain integer functions, usable on both sides.
#pragma once

#if defined(__HIPCC__) || defined(__HIP__)
#define BA_HD __host__ __device__ __forceinline__
#else
#define BA_HD inline
#endif

namespace ba {

// Division of a 32-bit unsigned number by a divisor fixed on the host (round-up multiplier of
// Granlund and Montgomery): n / d = (t + ((n - t) >> sh1)) >> sh2 with t = mulhi(n, mul); exact for
// every n.  A kernel divides by launch constants this way: a hardware division of wave-uniform
// numbers is some thirty scalar and vector instructions with two trips between the units.
struct FastDiv {
  unsigned mul, sh1, sh2;
};
inline FastDiv make_fast_div(unsigned d) {
  FastDiv f;
  unsigned l = 0;
  while ((1ull << l) < d) ++l;  // ceil(log2 d)
  f.mul = (unsigned)((((1ull << l) - d) << 32) / d + 1);
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l > 0 ? l - 1 : 0;
  return f;
}
BA_HD unsigned fast_div_u32(unsigned n, const FastDiv &f) {
  const unsigned t = (unsigned)(((unsigned long long)n * f.mul) >> 32);
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}
// divisors of split_tile_range, prepared on the host for the kernels
struct SplitDivs {
  FastDiv by_splits, by_two_splits;
};
inline SplitDivs make_split_divs(int n_splits) {
  SplitDivs d;
  d.by_splits = make_fast_div((unsigned)(n_splits > 0 ? n_splits : 1));
  d.by_two_splits = make_fast_div((unsigned)(n_splits > 0 ? 2 * n_splits : 2));
  return d;
}

struct TileRange {
  int begin, end;  // key tiles [begin, end) of a problem's walk (context tiles first, then the causal segment's)
};

// Key tiles of the causal segment that a row tile needs: up to the tile that holds the token of its
// last row (tokens and keys of a problem are the same rows, so token i sees keys 0..i).
BA_HD int causal_key_tiles(int last_tok, int tile_keys) { return last_tok / tile_keys + 1; }

// Split `split` of `n_splits` over a walk of n_ctx_tiles fully visible tiles followed by
// n_causal_tiles causal ones.  The splits are equal in tiles except that the walk is treated as
// `pad` tiles longer than it is: tiles of the causal segment cost more than context tiles (masks on
// the diagonal, the change of segment, the general path of the loop), so the split that ends with
// them gets fewer, and all splits of a launch end together.  Splits may be empty (few tiles).
// (nt < 2^26 and at most 32 splits: the products fit 32 bits)
// cuts (nullable): unequal shares, the list of the work item's KV head.  cuts[s] = where split s
// begins, as a fraction of the (padded) walk in units of 1 / 65536, cuts[0] = 0 <= cuts[1] <= ... <=
// cuts[n_splits] = 65536: the planner sizes the splits of a KV head by the speed of the XCD each of
// them runs on, so that all of them end together.
constexpr int kMaxSplits = 32;
// divs (nullable): the same quotients without hardware divisions (for the kernels).
BA_HD TileRange split_tile_range(int n_ctx_tiles, int n_causal_tiles, int n_splits, int split,
                                 const unsigned *cuts = nullptr, const SplitDivs *divs = nullptr) {
  const int nt = n_ctx_tiles + n_causal_tiles;
  int pad = 0;
  if (n_splits > 1) {
    const int a = (3 + n_causal_tiles) / 2;
    const int b = divs ? (int)fast_div_u32((unsigned)nt, divs->by_two_splits) : nt / (2 * n_splits);
    pad = a < b ? a : b;
  }
  const unsigned nt_v = (unsigned)(nt + pad);
  TileRange r;
  int e;
  if (cuts) {
    r.begin = (int)(((unsigned long long)nt_v * cuts[split]) >> 16);
    e = (int)(((unsigned long long)nt_v * cuts[split + 1]) >> 16);
  } else if (divs) {
    r.begin = (int)fast_div_u32(nt_v * (unsigned)split, divs->by_splits);
    e = (int)fast_div_u32(nt_v * (unsigned)(split + 1), divs->by_splits);
  } else {
    r.begin = (int)(nt_v * (unsigned)split / (unsigned)n_splits);
    e = (int)(nt_v * (unsigned)(split + 1) / (unsigned)n_splits);
  }
  r.end = e < nt ? e : nt;
  if (r.begin > r.end) r.begin = r.end;
  return r;
}

// Work item number -> (row tile, KV head, split) of a launch of the main core.  Row tiles run
// fastest (the row tiles of one (KV head, split) share every K/V tile); above them the (KV head,
// split) pairs are ordered by group of kv_group KV heads, then split, then head inside the group.
// With XCD-aware numbering of the workgroups (below) an XCD then runs a contiguous range of splits
// of ONE group of KV heads, so it fetches the query rows of that group only (at config 5, with
// groups of one: 256 KB instead of the whole 2 MB, which every XCD fetching at once at the start of
// a launch cost two microseconds); with larger groups the splits of a KV head lie on more than one
// XCD, so that their sizes can follow those XCDs' speeds (the planner weighs the two).
struct ItemOrder {
  int n_rowtiles, n_kv_heads, n_splits, kv_group;  // kv_group divides n_kv_heads
};
struct ItemDivs {
  FastDiv by_rowtiles, by_group_splits, by_group;
};
struct ItemCoords {
  int rowtile, kvh, split;
};
// (the default, when nothing is known of the XCDs' speeds: an XCD fetches as few query rows as the order allows)
constexpr int kDefaultKvGroup = 1;
inline ItemDivs make_item_divs(const ItemOrder &o) {
  ItemDivs d;
  d.by_rowtiles = make_fast_div((unsigned)(o.n_rowtiles > 0 ? o.n_rowtiles : 1));
  d.by_group_splits = make_fast_div((unsigned)(o.n_splits > 0 ? o.n_splits * o.kv_group : 1));
  d.by_group = make_fast_div((unsigned)o.kv_group);
  return d;
}
BA_HD ItemCoords item_coords(unsigned id, const ItemOrder &o, const ItemDivs *d = nullptr) {
  const unsigned gs = (unsigned)(o.n_splits * o.kv_group);
  const unsigned hi = d ? fast_div_u32(id, d->by_rowtiles) : id / (unsigned)o.n_rowtiles;
  const unsigned group = d ? fast_div_u32(hi, d->by_group_splits) : hi / gs;
  const unsigned rem = hi - group * gs;
  const unsigned split = d ? fast_div_u32(rem, d->by_group) : rem / (unsigned)o.kv_group;
  ItemCoords c;
  c.rowtile = (int)(id - hi * (unsigned)o.n_rowtiles);
  c.split = (int)split;
  c.kvh = (int)(group * (unsigned)o.kv_group + (rem - split * (unsigned)o.kv_group));
  return c;
}
BA_HD unsigned item_id(int rowtile, int kvh, int split, const ItemOrder &o) {
  const unsigned group = (unsigned)(kvh / o.kv_group), lo = (unsigned)(kvh % o.kv_group);
  return ((group * (unsigned)o.n_splits + (unsigned)split) * (unsigned)o.kv_group + lo) * (unsigned)o.n_rowtiles + (unsigned)rowtile;
}

// Which XCD runs workgroup `wg` of a launch: the dispatcher deals workgroup ids round-robin.
constexpr int kNumXcds = 8;
BA_HD int xcd_of_workgroup(unsigned wg) { return (int)(wg % kNumXcds); }
// The work item that workgroup `wg` of an n_wg-workgroup final-block launch takes: ids are regrouped
// so that each XCD (and its L2) gets a contiguous run of work items, which then share K/V tiles.
// runs: which run each XCD takes, four bits per XCD (XCD x takes run (runs >> 4x) & 7).  Neighbouring
// runs hold splits of the same KV heads (see ItemOrder), and only XCDs that share KV heads can be
// balanced against each other through the sizes of their splits, so the planner may put a slow XCD
// next to a fast one.  Anything but the identity needs runs of equal length (n_wg a multiple of 8).
constexpr unsigned kIdentityXcdRuns = 0x76543210u;
BA_HD bool xcd_runs_valid(unsigned runs, unsigned n_wg) {
  unsigned seen = 0;
  for (int x = 0; x < kNumXcds; ++x) seen |= 1u << ((runs >> (4 * x)) & 15u);
  return seen == 0xffu && (runs == kIdentityXcdRuns || n_wg % kNumXcds == 0);
}
BA_HD unsigned work_item_of_workgroup(unsigned wg, unsigned n_wg, unsigned runs = kIdentityXcdRuns) {
  const unsigned q = n_wg / kNumXcds, r = n_wg % kNumXcds, x = (runs >> (4 * (wg % kNumXcds))) & 7u;
  return x * q + (x < r ? x : r) + wg / kNumXcds;
}
// ... and the XCD that runs work item `item` of such a launch (the inverse, for the planner)
BA_HD int xcd_of_work_item(unsigned item, unsigned n_wg, unsigned runs = kIdentityXcdRuns) {
  const unsigned q = n_wg / kNumXcds, r = n_wg % kNumXcds;
  // run x holds items [x q + min(x, r), (x + 1) q + min(x + 1, r))
  const unsigned big = r * (q + 1);  // items in the r runs that hold q + 1 of them
  const unsigned run = item < big ? item / (q + 1) : r + (q ? (item - big) / q : 0);
  for (int x = 0; x < kNumXcds; ++x)
    if (((runs >> (4 * x)) & 7u) == run) return x;
  return (int)run;
}
// KV heads that get a cut list of their own when the splits are sized by XCD speed
constexpr int kMaxCutHeads = 8;

}  // namespace ba
