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

// Causal launches with few tiles per K/V head are ordered tile-major inside batches of K/V heads
// big enough to give every CU of an XCD about two workgroups (ATTN_CAUSAL_BATCH_WGS per XCD):
// the heaviest tiles of the whole batch start first and its lightest fill the gaps, instead of
// every head's light tiles being handed out before the next head's heavy ones.
#ifndef ATTN_CAUSAL_BATCH_WGS
#define ATTN_CAUSAL_BATCH_WGS 64
#endif

ATTN_HD inline AttnTileCoord attn_tile_coord_impl(int wg, int B, int Hq, int Hkv, int T, int causal) {
  const int G = Hq / Hkv;
  const int groups = B * Hkv;   // independent K/V heads
  const int W = G * T;          // workgroups that share one K/V head
  int xcd = 0, s = wg, lists = 1;
  if ((groups & 7) == 0) {
    xcd = wg & 7;
    s = wg >> 3;
    lists = 8;
  }
  int gl, tt, hg;  // K/V head within this XCD's list, tile rank (0 = first issued), query head within the group
  if (causal) {
    const int gx = groups / lists;  // K/V heads in this list
    const int per = (ATTN_CAUSAL_BATCH_WGS * (8 / lists) + W - 1) / W;  // K/V heads per batch
    const int pb = per < gx ? per : gx;
    const int batch = s / (pb * W), r = s % (pb * W);
    const int nb = gx - batch * pb < pb ? gx - batch * pb : pb;  // the last batch may be short
    tt = r / (nb * G);
    const int rem = r % (nb * G);
    gl = batch * pb + rem / G;
    hg = rem % G;
  } else {
    gl = s / W;
    const int inner = s % W;
    tt = inner / G;
    hg = inner % G;
  }
  const int group = gl * lists + xcd;
  AttnTileCoord c;
  c.b = group / Hkv;
  c.hq = (group % Hkv) * G + hg;
  c.t = causal ? (T - 1 - tt) : tt;
  return c;
}
