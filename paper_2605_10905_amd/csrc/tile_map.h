// Work decomposition shared by the host entry points and the device kernels.
//
// One workgroup owns one query tile (BM rows) of one (batch, query head).  The
// hardware hands consecutive workgroup ids to the 8 XCDs round-robin, and each
// XCD has a private L2.  All query tiles of the G = Hq/Hkv query heads that read
// one K/V head stream the same K/V bytes, so they are placed on ONE XCD and next
// to each other in dispatch order: K/V then comes from HBM once per XCD pass and
// from that XCD's L2 for every other workgroup.  This is the stand-in for the
// paper's cluster multicast / dynamic tile assignment (section 4.2), which has no
// hardware form on CDNA4.
//
// Causal tiles are issued heaviest first (the tile with the most visible keys),
// so the short tiles fill the tail of the launch.
#pragma once

#ifndef ATTN_HD
#define ATTN_HD __host__ __device__
#endif

struct AttnTileCoord {
  int b, hq, t;
};

ATTN_HD inline AttnTileCoord attn_tile_coord_impl(int wg, int B, int Hq, int Hkv, int T, int causal) {
  const int G = Hq / Hkv;
  const int groups = B * Hkv;   // independent K/V heads
  const int W = G * T;          // workgroups that share one K/V head
  int group, inner;
  if ((groups & 7) == 0) {
    const int xcd = wg & 7, s = wg >> 3;
    group = (s / W) * 8 + xcd;
    inner = s % W;
  } else {
    group = wg / W;
    inner = wg % W;
  }
  const int tt = inner / G, hg = inner % G;
  AttnTileCoord c;
  c.b = group / Hkv;
  c.hq = (group % Hkv) * G + hg;
  c.t = causal ? (T - 1 - tt) : tt;
  return c;
}
