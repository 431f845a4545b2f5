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
BA_HD TileRange split_tile_range(int n_ctx_tiles, int n_causal_tiles, int n_splits, int split) {
  const int nt = n_ctx_tiles + n_causal_tiles;
  int pad = 0;
  if (n_splits > 1) {
    const int a = (3 + n_causal_tiles) / 2, b = nt / (2 * n_splits);
    pad = a < b ? a : b;
  }
  const unsigned nt_v = (unsigned)(nt + pad);
  TileRange r;
  r.begin = (int)(nt_v * (unsigned)split / (unsigned)n_splits);
  const int e = (int)(nt_v * (unsigned)(split + 1) / (unsigned)n_splits);
  r.end = e < nt ? e : nt;
  if (r.begin > r.end) r.begin = r.end;
  return r;
}

}  // namespace ba
