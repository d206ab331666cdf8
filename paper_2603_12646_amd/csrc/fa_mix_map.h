// Workgroup-id -> tile map of the mixed-shape global kernel (head_dim 64, ONE sequence): plain
// integer arithmetic shared by the kernel (which evaluates it on the device from the sequence
// length it reads there) and the host (which sizes the launch for the worst length and whose
// tests walk every id on the CPU).
//
// A call of one sequence has T = ceil(n / 128) tiles of 128 rows per head and U = T * heads in
// all; 256 compute units hold two workgroups of this kernel each.  256-row workgroups ("A", two
// query blocks per wavefront) move half the K/V tile traffic per flop of 128-row ones ("B"), but
// an A workgroup alone on its unit runs at less than half rate, so a launch of A alone whose last
// round is thin, or just over one per unit, wastes much of that round.  The split:
//   U <= 512 or T < 2:  B only (at most two per unit anyway);
//   otherwise r = U / 1024 full rounds of A pairs (512 r workgroups), and for the R = U - 1024 r
//   tiles that remain
//       R <= 256:        R workgroups B (at most one per unit, beside the last A workgroups),
//       256 < R <= 512:  R / 2 more A (at most one per unit; measured 2-3 % faster than R times B),
//       512 < R <= 768:  R / 3 more A and as many (+ rounding) B: one pair A + B per unit,
//       R > 768:         R / 2 more A (nearly a full round).
// Measured on MI355X against the best single shape, 12 heads: 12K tokens (R = 128) +4 %, 24K
// (R = 256) +6 %, 28K (R = 640) +5 %, 8K x 20 heads (R = 256) +10 %, 8K x 12 heads (r = 0) +5-8 %.
// The A workgroups of a head cover its FIRST rows and are dealt to the heads as evenly as
// integers allow (head h gets floor(A (h+1) / heads) - floor(A h / heads)); their number is
// capped at heads * floor(T / 2) so that every head can hold its share.  B workgroups take the
// rows after them.
//
// Ids [0, ids_a) are the A range and come first, so that the dispatcher spreads the A workgroups
// over the units before the B workgroups follow; ids [ids_a, ids_a + ids_b) are the B range.
// Within a range ids are dealt round-robin to the 8 XCDs and every XCD takes a contiguous eighth
// of the range's (head, tile) list (XCD-aware order), or the list is walked in id order.  Ids
// without a tile are "spare": the kernel lets them zero-fill the tiles that lie wholly in the
// padding.  ids_a and ids_b must be multiples of 8 and at least the A / B totals of every
// length the call may see (fa_mix_ids).  Everything is 32-bit arithmetic: the callers keep
// T * heads <= 2^20 and heads <= 256, so that no product below exceeds 2^28.
#pragma once
#include <stdint.h>

#ifdef __HIPCC__
#define FA_HD __host__ __device__
#else
#define FA_HD
#endif

constexpr int kMixIdsB = 768;   // B workgroups never exceed 512 + rounding; spare ids live here too

struct FaMixTile {
  int kind;    // 0: nothing to do, 1: 256-row tile, 2: 128-row tile, 3: spare id
  int head;    // kinds 1, 2
  int q0;      // first query row (kinds 1, 2)
  int spare;   // kind 3: index of this id among the spare ids of the launch
  int spares;  // kind 3: number of spare ids
};

// number of 256-row workgroups for T = tiles, H = heads
FA_HD inline int fa_mix_a_total(int tiles, int H) {
  const int U = tiles * H;
  if (U <= 512 || tiles < 2) return 0;
  const int r = U / 1024, R = U - 1024 * r;
  const int a = 512 * r + (R > 768 ? R / 2 : (R > 512 ? R / 3 : (R > 256 && r > 0 ? R / 2 : 0)));
  const int cap = H * (tiles / 2);
  return a < cap ? a : cap;
}

FA_HD inline FaMixTile fa_mix_locate(int bid, bool map_xcd, int ids_a, int ids_b, int H, int tiles) {
  FaMixTile m = {0, 0, 0, 0, 0};
  const int a_tot = fa_mix_a_total(tiles, H);
  const int b_tot = tiles * H - 2 * a_tot;
  const bool range_a = bid < ids_a;
  const int j = range_a ? bid : bid - ids_a;
  const int tot = range_a ? a_tot : b_tot, ids = range_a ? ids_a : ids_b;
  const int per = (tot + 7) >> 3;      // list entries per XCD
  const int spare_a = map_xcd ? ids_a - 8 * ((a_tot + 7) >> 3) : ids_a - a_tot;
  const int spare_b = map_xcd ? ids_b - 8 * ((b_tot + 7) >> 3) : ids_b - b_tot;
  int t, spare = -1;
  if (map_xcd) {
    const int x = j & 7, p = j >> 3;   // XCD x owns entries [x per, x per + per) on ids x, x + 8, ...
    t = x * per + p;
    if (p >= per) spare = x * (ids / 8 - per) + (p - per);
    else if (t >= tot) return m;       // at most seven ids per range: the rounding of per
  } else {
    t = j;
    if (t >= tot) spare = t - tot;
  }
  if (spare >= 0) {
    m.kind = 3;
    m.spare = (range_a ? 0 : spare_a) + spare;
    m.spares = spare_a + spare_b;
    return m;
  }
  // 256-row workgroups of heads 0 .. h-1
  auto bnd = [&](int h) { return a_tot * h / H; };
  if (range_a) {
    int h = t * H / a_tot;
    while (h > 0 && bnd(h) > t) --h;
    while (h + 1 < H && bnd(h + 1) <= t) ++h;
    m.kind = 1;
    m.head = h;
    m.q0 = 256 * (t - bnd(h));
  } else {
    // 128-row tiles of heads 0 .. h-1: h * tiles - 2 bnd(h), nondecreasing in h
    auto pre = [&](int h) { return h * tiles - 2 * bnd(h); };
    int h = t * H / b_tot;
    while (h > 0 && pre(h) > t) --h;
    while (h + 1 < H && pre(h + 1) <= t) ++h;
    m.kind = 2;
    m.head = h;
    m.q0 = 256 * (bnd(h + 1) - bnd(h)) + 128 * (t - pre(h));
  }
  return m;
}

// Launch size for sequences of up to max_tiles tiles per head: ids_a (a multiple of 8), or -1 when
// some length would need more than kMixIdsB ids of 128-row workgroups (never, for heads <= 256).
inline int fa_mix_ids(int max_tiles, int H) {
  int a_max = 0;
  for (int t = 0; t <= max_tiles; ++t) {
    const int a = fa_mix_a_total(t, H);
    const int b = t * H - 2 * a;
    if (8 * ((b + 7) / 8) >= kMixIdsB) return -1;   // keeps at least one spare id in the B range
    a_max = a > a_max ? a : a_max;
  }
  return 8 * ((a_max + 7) / 8);
}
