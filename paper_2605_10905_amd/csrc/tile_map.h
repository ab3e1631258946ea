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

// What the map needs that does not depend on the workgroup id, made once per launch on the host
// (divisions by these values are then a multiply-high and one correction in the kernel, instead of
// a generic integer division each: the forward kernel maps a tile before it can request its first
// byte, and again at every seam between the tiles of a resident workgroup).
struct AttnTileMap {
  int G, Hkv, T, W, lists, causal;
  int gx, pb;                               // causal: K/V heads per list, K/V heads per batch
  unsigned m_W, m_G, m_Hkv, m_pbW, m_pbG;   // floor(2^32 / divisor)
};

ATTN_HD inline unsigned attn_div_magic(int d) { return d > 1 ? (unsigned)(0x100000000ull / (unsigned)d) : 0xffffffffu; }

// n / d for 0 <= n < 2^31, d >= 1, m = attn_div_magic(d): the estimate is the quotient or one less
ATTN_HD inline int attn_fast_div(int n, int d, unsigned m, int* rem) {
  int q = (int)(((unsigned long long)(unsigned)n * m) >> 32);
  int r = n - q * d;
  if (r >= d) {
    ++q;
    r -= d;
  }
  *rem = r;
  return q;
}

ATTN_HD inline AttnTileMap attn_tile_map_make(int B, int Hq, int Hkv, int T, int causal) {
  AttnTileMap m;
  m.G = Hq / Hkv;
  m.Hkv = Hkv;
  m.T = T;
  m.W = m.G * T;  // workgroups that share one K/V head
  const int groups = B * Hkv;  // independent K/V heads
  m.lists = (groups & 7) == 0 ? 8 : 1;
  m.causal = causal;
  m.gx = groups / m.lists;
  const int per = (ATTN_CAUSAL_BATCH_WGS * (8 / m.lists) + m.W - 1) / m.W;
  m.pb = per < m.gx ? per : m.gx;
  m.m_W = attn_div_magic(m.W);
  m.m_G = attn_div_magic(m.G);
  m.m_Hkv = attn_div_magic(Hkv);
  m.m_pbW = attn_div_magic(m.pb * m.W);
  m.m_pbG = attn_div_magic(m.pb * m.G);
  return m;
}

ATTN_HD inline AttnTileCoord attn_tile_coord_map(int wg, const AttnTileMap& m) {
  int xcd = 0, s = wg;
  if (m.lists == 8) {
    xcd = wg & 7;
    s = wg >> 3;
  }
  int gl, tt, hg;  // K/V head within this XCD's list, tile rank (0 = first issued), query head within the group
  if (m.causal) {
    int r, rem;
    const int batch = attn_fast_div(s, m.pb * m.W, m.m_pbW, &r);
    const int left = m.gx - batch * m.pb;  // the last batch may be short
    if (left >= m.pb) {
      tt = attn_fast_div(r, m.pb * m.G, m.m_pbG, &rem);
    } else {
      tt = r / (left * m.G);
      rem = r % (left * m.G);
    }
    gl = batch * m.pb + attn_fast_div(rem, m.G, m.m_G, &hg);
  } else {
    int inner;
    gl = attn_fast_div(s, m.W, m.m_W, &inner);
    tt = attn_fast_div(inner, m.G, m.m_G, &hg);
  }
  const int group = gl * m.lists + xcd;
  AttnTileCoord c;
  int hk;
  c.b = attn_fast_div(group, m.Hkv, m.m_Hkv, &hk);
  c.hq = hk * m.G + hg;
  c.t = m.causal ? (m.T - 1 - tt) : tt;
  return c;
}

ATTN_HD inline AttnTileCoord attn_tile_coord_impl(int wg, int B, int Hq, int Hkv, int T, int causal) {
  return attn_tile_coord_map(wg, attn_tile_map_make(B, Hq, Hkv, T, causal));
}
