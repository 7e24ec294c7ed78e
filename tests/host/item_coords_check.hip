// Host-side check of the item -> (segment, query block, head, sequence, head sub-group, prefix piece)
// mapping of the prefill and dQ kernels (item_coords in segattn_work.h), over many launch shapes:
//   * the form with host-prepared multiply-shift divisors equals the form with plain divisions;
//   * the map is one-to-one onto the launch's items: every (segment, block, head, sequence,
//     sub-group[, piece]) exactly once;
//   * the items of the heads listed first (full-history heads) come first, longest first.
// Prints "ok <launches> <items>" or the first failure.  Pure host code: needs no GPU.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "segattn_work.h"

using namespace segattn;

static long long gcd_ll(long long x, long long y) {
  while (y) {
    const long long t = x % y;
    x = y;
    y = t;
  }
  return x;
}
static int coprime_stride(long long groups) {  // the smallest number >= groups / 8 coprime to groups
  if (groups <= 1) return 1;
  long long s = groups / 8 > 0 ? groups / 8 : 1;
  while (gcd_ll(s, groups) != 1) ++s;
  return (int)s;
}

static long long launches = 0, items_checked = 0;

static void fail(const char *what, const Problem &p, const PrefillArgs &a, int hw, long long bid) {
  printf("FAILED: %s (B=%d Hkv=%d n_past=%d g=%d heads/wg=%d n_seg=%d nqb=%d parts=%d sub=%d packed=%d retrieved=%d) at item %lld\n",
         what, p.B, p.Hkv, p.n_past, p.g, hw, a.n_seg, a.q_blocks_per_seg, a.parts, a.sub_groups, a.cu_seqlens != nullptr,
         a.ret_k != nullptr, bid);
  exit(1);
}

static void check_launch(int B, int Hkv, int n_past, int g, int hw, int n_seg, int nqb, int parts, int sub, bool packed,
                         bool retrieved) {
  static int dummy_cu[2];
  static unsigned short dummy_k[2];
  static unsigned char dummy_cache[8];
  Problem p;
  memset(&p, 0, sizeof(p));
  p.B = B;
  p.Hkv = Hkv;
  p.n_past = n_past;
  p.g = g;
  p.Hq = Hkv * g;
  for (int i = 0; i < Hkv; ++i) p.order[i] = i;
  PrefillArgs a;
  memset(&a, 0, sizeof(a));
  a.n_seg = n_seg;
  a.q_blocks_per_seg = nqb;
  a.parts = parts;
  a.sub_groups = sub;
  if (packed) a.cu_seqlens = dummy_cu;
  if (retrieved) a.ret_k = dummy_k;
  if (parts > 1) a.cache = dummy_cache;  // prefix pieces exist in the stateful form only
  const int nhs = g / hw;
  const int n_first = retrieved ? 0 : n_past;
  const int n_other = Hkv - n_first;
  const int eff_parts = parts > 1 ? parts : 1;
  const long long past_items = (long long)B * n_first * nhs * n_seg * nqb * eff_parts;
  const long long grid = past_items + (long long)B * n_other * nhs * n_seg * nqb;
  if (grid <= 0 || grid >= (1ll << 31)) return;
  a.pair_stride = coprime_stride((long long)B * n_other * nhs * n_seg);
  a.grid_items = (int)grid;
  PrefillArgs fast = a;
  prepare_resolve_divs(p, fast, hw, grid);
  if (!fast.dv.ok) fail("divisors were not prepared", p, a, hw, -1);
  std::vector<unsigned char> seen((size_t)grid, 0);
  long long last_gq = 1ll << 40;
  for (long long bid = 0; bid < grid; ++bid) {
    const ItemCoords x = item_coords(p, a, (int)bid, (int)grid, hw);
    const ItemCoords y = item_coords(p, fast, (int)bid, (int)grid, hw);
    if (x.seg != y.seg || x.qblk != y.qblk || x.hidx != y.hidx || x.b != y.b || x.hs != y.hs || x.part != y.part)
      fail("prepared divisors disagree with plain division", p, a, hw, bid);
    if (x.seg < 0 || x.seg >= n_seg || x.qblk < 0 || x.qblk >= nqb || x.b < 0 || x.b >= B || x.hs < 0 || x.hs >= nhs ||
        x.hidx < 0 || x.hidx >= Hkv || x.part < 0 || x.part >= eff_parts)
      fail("coordinate out of range", p, a, hw, bid);
    const bool first = x.hidx < n_first;
    if (first != (bid < past_items)) fail("heads listed first must own the first items", p, a, hw, bid);
    if (!first && x.part != 0) fail("only full-history heads have prefix pieces", p, a, hw, bid);
    long long id;  // a dense index of the coordinates inside their half of the launch
    if (first) {
      id = ((((long long)x.seg * nqb + x.qblk) * B + x.b) * n_first + x.hidx) * nhs + x.hs;
      id = id * eff_parts + x.part;
      const long long gq = (long long)x.seg * nqb + x.qblk;
      if (gq > last_gq) fail("full-history items must come longest first", p, a, hw, bid);
      last_gq = gq;
    } else {
      id = past_items + ((((long long)x.seg * nqb + x.qblk) * B + x.b) * n_other + (x.hidx - n_first)) * nhs + x.hs;
    }
    if (id < 0 || id >= grid || seen[(size_t)id]) fail("an item's coordinates appear twice", p, a, hw, bid);
    seen[(size_t)id] = 1;
  }
  ++launches;
  items_checked += grid;
}

int main() {
  const int Bs[] = {1, 2, 3, 12};
  const int segs[] = {1, 2, 5, 32};
  const int nqbs[] = {1, 3, 8, 16, 64};
  for (int B : Bs)
    for (int Hkv : {1, 2, 8})
      for (int n_past = 0; n_past <= Hkv; n_past += (Hkv > 2 ? 3 : 1))
        for (int g : {1, 4, 6})
          for (int hw : {1, 2, 4}) {
            if (g % hw) continue;
            for (int n_seg : segs)
              for (int nqb : nqbs) {
                for (int sub : {1, 2, 4, 8}) {
                  if (nqb % sub) continue;
                  check_launch(B, Hkv, n_past, g, hw, n_seg, nqb, 1, sub, false, false);
                }
                check_launch(B, Hkv, n_past, g, hw, n_seg, nqb, 1, 1, true, false);   // packed batch: rotated assignment
                check_launch(B, Hkv, n_past, g, hw, n_seg, nqb, 1, 1, false, true);   // retrieved prefixes: one common list
                if (n_past > 0 && n_seg == 1)
                  for (int parts : {2, 3, 4}) check_launch(B, Hkv, n_past, g, hw, 1, nqb, parts, 1, false, false);
              }
          }
  // the benchmark's shapes: 128K tokens, 32 / 8 heads, two full-history heads, 64-row blocks
  check_launch(1, 8, 2, 4, 4, 32, 64, 1, 1, false, false);
  check_launch(12, 8, 2, 4, 4, 8, 64, 1, 1, true, false);
  check_launch(1, 8, 4, 4, 4, 32, 64, 1, 1, false, true);
  check_launch(1, 2, 0, 4, 4, 1, 256, 1, 4, false, false);
  printf("ok %lld %lld\n", launches, items_checked);
  return 0;
}
