// Host: the plan section of the row-band kernel (bsp_rows.hip), see bsp_plan.h.
// Groups block rows into strips by the overlap of their kept columns, lists each strip's
// contraction as column steps and writes the weights in matrix-core operand order.
#include "bsp.h"
#include "bsp_plan.h"

#include <algorithm>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

namespace {

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

struct Bits {
  int words = 0;
  std::vector<uint64_t> w;  // [rows][words]
  const uint64_t* row(int r) const { return &w[(size_t)r * words]; }
  uint64_t* row(int r) { return &w[(size_t)r * words]; }
};

inline int popcount_or(const uint64_t* a, const uint64_t* b, int n) {
  int c = 0;
  for (int i = 0; i < n; ++i) c += __builtin_popcountll(a[i] | b[i]);
  return c;
}
inline int popcount1(const uint64_t* a, int n) {
  int c = 0;
  for (int i = 0; i < n; ++i) c += __builtin_popcountll(a[i]);
  return c;
}

// Kept units of a group of rows.
int group_union(const Bits& b, const std::vector<int>& g, std::vector<uint64_t>& u) {
  std::fill(u.begin(), u.end(), 0);
  for (int r : g)
    for (int i = 0; i < b.words; ++i) u[i] |= b.row(r)[i];
  return popcount1(u.data(), b.words);
}

// Block rows -> strips of `rps` rows with small unions: greedy (heaviest unplaced row
// first, then the rows that add the fewest new columns), then pairwise swaps between
// strips while the sum of the unions drops.
// Groups rows first .. first + count - 1 only (a window of output channels), or all of them.
std::vector<std::vector<int>> group_rows(const Bits& bits, int nbr, int rps, int first = 0, int count = -1) {
  std::vector<std::vector<int>> groups;
  if (count < 0) count = nbr - first;
  if (rps == 1) {
    for (int r = first; r < first + count; ++r) groups.push_back({r});
    return groups;
  }
  const int W = bits.words;
  std::vector<int> order(count);
  std::iota(order.begin(), order.end(), first);
  std::vector<int> pc(nbr, 0);
  for (int r = first; r < first + count; ++r) pc[r] = popcount1(bits.row(r), W);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return pc[a] > pc[b]; });
  std::vector<char> used(nbr, 0);
  std::vector<uint64_t> u(W);
  for (int oi = 0; oi < count; ++oi) {
    const int seed = order[oi];
    if (used[seed]) continue;
    used[seed] = 1;
    std::vector<int> g = {seed};
    std::copy(bits.row(seed), bits.row(seed) + W, u.begin());
    while ((int)g.size() < rps) {
      int best = -1, best_cost = std::numeric_limits<int>::max();
      for (int oj = 0; oj < count; ++oj) {
        const int r = order[oj];
        if (used[r]) continue;
        const int cost = popcount_or(u.data(), bits.row(r), W) * 4096 - pc[r];
        if (cost < best_cost) best_cost = cost, best = r;
      }
      if (best < 0) break;
      used[best] = 1;
      g.push_back(best);
      for (int i = 0; i < W; ++i) u[i] |= bits.row(best)[i];
    }
    groups.push_back(g);
  }
  // pairwise swaps
  const int ng = (int)groups.size();
  std::vector<int> cost(ng);
  for (int a = 0; a < ng; ++a) cost[a] = group_union(bits, groups[a], u);
  std::vector<uint64_t> ua(W), ub(W);
  const int64_t work = (int64_t)ng * ng * W * rps * rps;
  const int passes = work > (int64_t)4e8 ? 0 : work > (int64_t)5e7 ? 2 : 8;
  for (int pass = 0; pass < passes; ++pass) {
    bool any = false;
    for (int a = 0; a < ng; ++a)
      for (int b = a + 1; b < ng; ++b) {
        for (size_t i = 0; i < groups[a].size(); ++i)
          for (size_t j = 0; j < groups[b].size(); ++j) {
            std::swap(groups[a][i], groups[b][j]);
            const int ca = group_union(bits, groups[a], ua), cb = group_union(bits, groups[b], ub);
            if (ca + cb < cost[a] + cost[b]) {
              cost[a] = ca;
              cost[b] = cb;
              any = true;
            } else {
              std::swap(groups[a][i], groups[b][j]);
            }
          }
      }
    if (!any) break;
  }
  for (auto& g : groups) std::sort(g.begin(), g.end());
  return groups;
}

}  // namespace

bool bsp_rows_wanted(int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                     int32_t dtype) {
  (void)bo;
  (void)bi;
  if (dtype != BSP_BF16) return false;
  if ((I % 8) != 0 || (O % 8) != 0) return false;
  if (H > BSP_ROWS_MAXH || K > 15) return false;
  // very large fully-connected layers are served from the compressed rows themselves
  if ((int64_t)O * I * H * K > (int64_t)48 << 20) return false;
  return true;
}

// Fills `sec` (words) with the section; with payload == nullptr the weights are left zero
// (the size is the same).  `base_words` is the section's offset in the plan, a multiple of 4.
int bsp_rows_section(const int32_t* row_ptr, const int32_t* col_idx, const uint16_t* payload,
                     int32_t O, int32_t H, int32_t K, int32_t I, int32_t bo, int32_t bi,
                     std::vector<int32_t>* sec) {
  const int nbr = (int)cdiv(O, bo);
  const int rps = BSP_STRIP / bo;              // block rows per strip: 2, 4, 1
  const int cw = bi == 4 ? 4 : 8;              // channels per contraction item
  const int ips = 32 / cw;                     // items per column step: 4 or 8
  const int nunits = (int)cdiv(I, cw);         // contraction units (channel groups) of the layer
  const int slab = bsp_rows_slab(I, H, K, cw);
  const int upslab = slab / cw;                // units per slab
  const int nslabs = (int)cdiv(nunits, upslab);
  const int64_t HK = (int64_t)H * K;
  const int64_t blk_elems = (int64_t)bo * bi * HK;

  // kept units per block row
  Bits bits;
  bits.words = (int)cdiv(nunits, 64);
  bits.w.assign((size_t)nbr * bits.words, 0);
  for (int r = 0; r < nbr; ++r)
    for (int64_t n = row_ptr[r]; n < row_ptr[r + 1]; ++n) {
      const int c = col_idx[n];
      const int u0 = c * bi / cw, u1 = std::min<int>(nunits, (c + 1) * bi / cw);
      for (int u = u0; u < u1; ++u) bits.row(r)[u >> 6] |= 1ull << (u & 63);
    }
  // Pointwise layers: rows are grouped within windows of 64 output channels, and the strips
  // of a window stay together, in window order: a workgroup that takes whole windows then
  // produces whole 128-byte lines of every output pixel.
  const int wstrips = bsp_rows_window(H, K);
  std::vector<std::vector<int>> groups;
  if (wstrips == 0) {
    groups = group_rows(bits, nbr, rps);
  } else {
    const int wrows = wstrips * rps;
    for (int r0 = 0; r0 < nbr; r0 += wrows) {
      std::vector<std::vector<int>> g = group_rows(bits, nbr, rps, r0, std::min(wrows, nbr - r0));
      groups.insert(groups.end(), g.begin(), g.end());
    }
  }
  const int nstrips = (int)groups.size();

  // per strip: kept units (union), column steps per slab
  std::vector<std::vector<int>> units(nstrips);
  std::vector<int> steps_of(nstrips, 0);
  std::vector<uint64_t> u(bits.words);
  for (int t = 0; t < nstrips; ++t) {
    group_union(bits, groups[t], u);
    int slab_items = 0, cur = 0;
    for (int x = 0; x < nunits; ++x) {
      if (!((u[x >> 6] >> (x & 63)) & 1)) continue;
      const int sl = x / upslab;
      if (sl != cur) {
        steps_of[t] += (int)cdiv((int64_t)slab_items * K, ips);
        slab_items = 0;
        cur = sl;
      }
      units[t].push_back(x);
      ++slab_items;
    }
    steps_of[t] += (int)cdiv((int64_t)slab_items * K, ips);
  }
  // heaviest strips first: a workgroup takes consecutive strips, which then cost alike
  std::vector<int> order(nstrips);
  std::iota(order.begin(), order.end(), 0);
  if (wstrips == 0)
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return steps_of[a] > steps_of[b]; });

  int64_t ncs = 0;
  for (int t = 0; t < nstrips; ++t) ncs += steps_of[t];
  const int64_t off_rstrip = BSP_ROWS_HEADER_WORDS;
  const int64_t off_rslab = off_rstrip + (int64_t)nstrips * 4;
  const int64_t off_rdesc = off_rslab + (int64_t)nstrips * (nslabs + 1);
  const int64_t off_rfrag = (off_rdesc + ncs * 4 + 3) & ~int64_t(3);
  const int64_t total = off_rfrag + ncs * H * 64 * 4;
  if (total > std::numeric_limits<int32_t>::max() / 2) return BSP_ERR_SHAPE;
  sec->assign((size_t)total, 0);
  int32_t* s = sec->data();
  s[BSP_ROWS_NSTRIPS_W] = nstrips;
  s[BSP_ROWS_SLAB_W] = slab;
  s[BSP_ROWS_NSLABS_W] = nslabs;
  s[BSP_ROWS_NCS_W] = (int32_t)ncs;
  s[BSP_ROWS_RESERVED_W] = 0;
  s[BSP_ROWS_OFF_STRIP_W] = (int32_t)off_rstrip;
  s[BSP_ROWS_OFF_SLAB_W] = (int32_t)off_rslab;
  s[BSP_ROWS_OFF_DESC_W] = (int32_t)off_rdesc;
  s[BSP_ROWS_OFF_FRAG_W] = (int32_t)off_rfrag;
  s[BSP_ROWS_CW_W] = cw;
  s[BSP_ROWS_WINDOW_W] = wstrips;
  int32_t* rstrip = s + off_rstrip;
  int32_t* rslab = s + off_rslab;
  int32_t* rdesc = s + off_rdesc;
  uint16_t* rfrag = (uint16_t*)(s + off_rfrag);

  // block (row, column) -> position in the payload, for the rows of one strip
  std::vector<int32_t> pos;
  const int nbc = (int)cdiv(I, bi);
  int64_t cs = 0;
  int max_steps = 0, max_strip_steps = 0;
  int64_t kept_items = 0, union_items = 0;
  for (int ti = 0; ti < nstrips; ++ti) {
    const int t = order[ti];
    const std::vector<int>& g = groups[t];
    for (int q = 0; q < 4; ++q) {
      const int srow = 4 * q;  // strip row of this lane group's first output row
      const int member = srow / bo;
      int32_t chan = -1;
      if (member < (int)g.size()) {
        chan = g[member] * bo + srow % bo;
        if (chan + 4 > O) chan = -1;  // O is a multiple of 8: a group of four is all in or all out
      }
      rstrip[ti * 4 + q] = chan;
    }
    pos.assign((size_t)rps * nbc, -1);
    for (size_t m = 0; m < g.size(); ++m)
      for (int64_t n = row_ptr[g[m]]; n < row_ptr[g[m] + 1]; ++n) {
        const int cn = col_idx[n];
        pos[m * nbc + cn] = (int32_t)n;
        kept_items += std::min<int64_t>(nunits, (int64_t)(cn + 1) * bi / cw) - (int64_t)cn * bi / cw;
      }
    union_items += (int64_t)units[t].size();
    size_t e = 0;
    const int64_t strip_first = cs;
    for (int sl = 0; sl < nslabs; ++sl) {
      rslab[ti * (nslabs + 1) + sl] = (int32_t)cs;
      const size_t e0 = e;
      while (e < units[t].size() && units[t][e] / upslab == sl) ++e;
      const int64_t items = (int64_t)(e - e0) * K;
      const int64_t nst = cdiv(items, ips);
      if (nst > max_steps) max_steps = (int)nst;
      for (int64_t st = 0; st < nst; ++st) {
        for (int q = 0; q < 4; ++q) {
          int32_t d = 0;
          for (int h = 0; h < ips / 4; ++h) {  // one item per lane group (cw 8) or two (cw 4)
            const int64_t it = st * ips + q * (ips / 4) + h;
            int32_t code = 0;
            if (it < items) {
              const int unit = units[t][e0 + (size_t)(it / K)];
              const int dx = (int)(it % K);
              code = (unit - sl * upslab) | (dx << 8);
            }
            d |= code << (16 * h);
          }
          rdesc[(cs + st) * 4 + q] = d;
        }
        if (!payload) continue;
        for (int dy = 0; dy < H; ++dy)
          for (int lane = 0; lane < 64; ++lane) {
            const int j = lane & 15, q = lane >> 4;
            uint16_t* dst = rfrag + (((cs + st) * H + dy) * 64 + lane) * 8;
            const int member = j / bo, r = j % bo;
            if (member >= (int)g.size()) continue;
            for (int h = 0; h < ips / 4; ++h) {
              const int64_t it = st * ips + q * (ips / 4) + h;
              if (it >= items) continue;
              const int unit = units[t][e0 + (size_t)(it / K)];
              const int dx = (int)(it % K);
              const int ch = unit * cw;          // first input channel of the item
              const int bc = ch / bi;
              const int32_t n = pos[(size_t)member * nbc + bc];
              if (n < 0) continue;
              const uint16_t* src = payload + (int64_t)n * blk_elems +
                                    ((int64_t)r * HK + (int64_t)dy * K + dx) * bi + ch % bi;
              std::memcpy(dst + h * cw, src, (size_t)cw * 2);
            }
          }
      }
      cs += nst;
    }
    rslab[ti * (nslabs + 1) + nslabs] = (int32_t)cs;
    if (cs - strip_first > max_strip_steps) max_strip_steps = (int)(cs - strip_first);
  }
  s[BSP_ROWS_MAXSTEPS_W] = max_steps;
  s[BSP_ROWS_MAXSTRIPSTEPS_W] = max_strip_steps;
  s[BSP_ROWS_KEPT_ITEMS_W] = (int32_t)std::min<int64_t>(kept_items, std::numeric_limits<int32_t>::max());
  s[BSP_ROWS_UNION_ITEMS_W] = (int32_t)std::min<int64_t>(union_items, std::numeric_limits<int32_t>::max());
  return BSP_OK;
}
