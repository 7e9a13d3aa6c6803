// Device-side statement of the cache partition (Section 4.1, Eq. 1) and of the rows the per-row
// eviction protects (Section 4.2), shared by the ranking and the V-cosine kernels.
#pragma once

#include "adsa.h"

namespace adsa {

// Geometry of one sequence's query for its current decode step s.
struct QueryCell {
  int P;              // grid origin (absolute position of image token 0)
  int n_keep_prefix;  // pinned leading positions
  int jq;             // image index of the query token (s - 1)
  int r, col;         // its grid cell
  int W, R, w;
  int recent_m;       // > 0: 1-D window of the m most recent image tokens instead of the 2-D one
};

__device__ __forceinline__ QueryCell make_query_cell(const adsa_seq& sq, int s, int W, int R, int w,
                                                     int recent_m = 0) {
  QueryCell c;
  c.P = sq.grid_origin; c.n_keep_prefix = sq.n_keep_prefix; c.jq = s - 1;
  c.r = s >= 1 ? c.jq / W : 0;
  c.col = s >= 1 ? c.jq - c.r * W : 0;
  c.W = W; c.R = R; c.w = w; c.recent_m = recent_m;
  return c;
}

// Attention-time partition: 0 = pinned prefix or local window (always attended), 1 = candidate
// ("previous"), -1 = entry newer than the query (malformed state).
__device__ __forceinline__ int select_class(const QueryCell& c, int pos) {
  if (pos < c.n_keep_prefix) return 0;
  if (pos < c.P) return 1;
  const int j = pos - c.P;
  if (j > c.jq) return -1;
  if (c.recent_m > 0) return j > c.jq - c.recent_m ? 0 : 1;
  const int rj = j / c.W, cj = j - rj * c.W;
  const int dc = cj > c.col ? cj - c.col : c.col - cj;
  const bool local = (rj == c.r) || (rj >= c.r - c.R && rj < c.r && dc <= c.w);
  return local ? 0 : 1;
}

// Eviction-time partition at the end of row r: 0 = pinned prefix or a token some window of the next
// row needs -- the last R completed rows (2-D window) or the m - 1 most recent tokens (1-D window: the
// next row's first query, jq + 1, reaches back furthest, to j > jq + 1 - m) --, 1 = competes for the budget.
__device__ __forceinline__ int evict_class(const QueryCell& c, int pos) {
  if (pos < c.n_keep_prefix) return 0;
  if (pos >= c.P) {
    const int j = pos - c.P;
    if (c.recent_m > 0) return j > c.jq + 1 - c.recent_m ? 0 : 1;
    const int rj = j / c.W;
    if (rj >= c.r - c.R + 1 && rj <= c.r) return 0;
  }
  return 1;
}

__device__ __forceinline__ bool is_row_end(int s, int grid_h, int W) {
  return s >= 1 && s <= grid_h * W && ((s - 1) % W == W - 1);
}

}  // namespace adsa
