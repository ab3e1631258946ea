// Work decomposition of the bf16 GEMM: one workgroup owns one BM x BN tile of C.
//
// The hardware hands consecutive workgroup ids to the 8 XCDs round-robin and each XCD has a
// private L2, so the tile list is cut into 8 contiguous pieces, one per XCD, and the list
// itself walks C in bands of GEMM_GROUP tile rows, column by column inside a band: the
// workgroups that are resident on one XCD at a time then cover a few tile rows x a few tile
// columns and share their A and B panels through that XCD's L2.  (The paper's GEMM gets the
// same reuse from cluster multicast and cluster launch control, section 4.2.)
#pragma once

#ifndef GEMM_HD
#define GEMM_HD __host__ __device__
#endif

#define GEMM_GROUP 4

struct GemmTileCoord {
  int tm, tn;
};

GEMM_HD inline GemmTileCoord gemm_tile_coord_impl(int wg, int tiles_m, int tiles_n) {
  const int T = tiles_m * tiles_n;
  const int xcd = wg & 7, idx = wg >> 3;
  const int base = T >> 3, rem = T & 7;
  // XCD x owns base + (x < rem) consecutive list entries, which is also how many ids it is handed
  const int L = xcd * base + (xcd < rem ? xcd : rem) + idx;
  const int width = GEMM_GROUP * tiles_n;
  const int band = L / width, in = L % width;
  const int first = band * GEMM_GROUP;
  const int rows = tiles_m - first < GEMM_GROUP ? tiles_m - first : GEMM_GROUP;
  GemmTileCoord c;
  c.tm = first + in % rows;
  c.tn = in / rows;
  return c;
}
