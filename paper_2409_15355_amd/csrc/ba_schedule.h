// Arithmetic of the schedule that the host planner and the kernels must agree on, written once:
// which key tiles a work item walks.  Plain integer functions, usable on both sides.
#pragma once

#if defined(__HIPCC__) || defined(__HIP__)
#define BA_HD __host__ __device__ __forceinline__
#else
#define BA_HD inline
#endif

namespace ba {

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
// cuts (nullable): unequal shares.  cuts[s] = where split s begins, as a fraction of the (padded) walk
// in units of 1 / 65536, cuts[0] = 0 <= cuts[1] <= ... <= cuts[n_splits] = 65536: the planner sizes
// the splits by the speed of the XCD each of them runs on, so that all of them end together.
constexpr int kMaxSplits = 32;
BA_HD TileRange split_tile_range(int n_ctx_tiles, int n_causal_tiles, int n_splits, int split,
                                 const unsigned *cuts = nullptr) {
  const int nt = n_ctx_tiles + n_causal_tiles;
  int pad = 0;
  if (n_splits > 1) {
    const int a = (3 + n_causal_tiles) / 2, b = nt / (2 * n_splits);
    pad = a < b ? a : b;
  }
  const unsigned nt_v = (unsigned)(nt + pad);
  TileRange r;
  int e;
  if (cuts) {
    r.begin = (int)(((unsigned long long)nt_v * cuts[split]) >> 16);
    e = (int)(((unsigned long long)nt_v * cuts[split + 1]) >> 16);
  } else {
    r.begin = (int)(nt_v * (unsigned)split / (unsigned)n_splits);
    e = (int)(nt_v * (unsigned)(split + 1) / (unsigned)n_splits);
  }
  r.end = e < nt ? e : nt;
  if (r.begin > r.end) r.begin = r.end;
  return r;
}

// Which XCD runs workgroup `wg` of a launch: the dispatcher deals workgroup ids round-robin.
constexpr int kNumXcds = 8;
BA_HD int xcd_of_workgroup(unsigned wg) { return (int)(wg % kNumXcds); }
// The work item that workgroup `wg` of an n_wg-workgroup final-block launch takes: ids are regrouped
// so that each XCD (and its L2) gets a contiguous run of work items, which then share K/V tiles.
BA_HD unsigned work_item_of_workgroup(unsigned wg, unsigned n_wg) {
  const unsigned q = n_wg / kNumXcds, r = n_wg % kNumXcds, x = wg % kNumXcds;
  return x * q + (x < r ? x : r) + wg / kNumXcds;
}

}  // namespace ba
