// Host-side work list of the persistent prefill kernel: items, and one chain of items per workgroup.
#pragma once

#include <algorithm>
#include <vector>

#include "internal.h"

namespace spd {

// One workgroup per compute unit walks a chain of work items.  Workgroup b runs on XCD b % xcds
// (round-robin dispatch), and each XCD has its own L2, so all items that read the same K, V - the
// query tiles and head groups of one (request, KV head) "unit" - go to chains of the same XCD.
// Units are spread over the XCDs longest-first; inside an XCD the items are dealt longest-first onto
// the least-loaded chain (weight = KV tiles to visit + a fixed per-item cost: measured, an item costs what
// four tiles cost beyond its own, in query loads, output stores and a first tile that sets the softmax
// reference), and every chain is
// ordered by unit, so that the chains of an XCD work on the same unit at about the same time.
// With fewer units than XCDs the items themselves are dealt round-robin.
// n_blocks == 0 asks for one workgroup per item instead (chains of length one, handed out by the
// hardware in launch order: the XCDs' queues interleaved, each queue heaviest unit first): for
// partitions on which a launch of exactly one workgroup per compute unit does not get one compute
// unit each.
constexpr long ITEM_COST_TILES = 4;

inline void build_prefill_chains(const int32_t* cu_seqlens, const int32_t* prefix_lens, const int32_t* kv_cu, int n_req,
                                 int H, int Hkv, int xcds, int n_blocks, std::vector<PrefillWork>& work,
                                 std::vector<int32_t>& chain) {
  const int G = H / Hkv, hb = prefill_heads_per_block(G), bm = prefill_block_m(G), groups = G / hb;
  struct Item { PrefillWork w; long weight; int unit; };
  struct Unit { long weight; std::vector<Item> items; };
  std::vector<Unit> units;
  for (int r = 0; r < n_req; ++r) {
    const int32_t row0 = cu_seqlens[r], len = cu_seqlens[r + 1] - row0;
    const int32_t q_off = prefix_lens ? prefix_lens[r] : 0, kv_row0 = prefix_lens ? kv_cu[r] : row0;
    const int tiles = (len + bm - 1) / bm;
    for (int g = 0; g < Hkv; ++g) {
      Unit u{0, {}};
      for (int t = tiles - 1; t >= 0; --t)
        for (int hg = 0; hg < groups; ++hg) {
          const long kv_tiles = (q_off + std::min<long>(len, (long)(t + 1) * bm) + 63) / 64;
          u.items.push_back(Item{PrefillWork{row0, len, t, g * G + hg * hb, kv_row0, q_off}, kv_tiles + ITEM_COST_TILES, (int)units.size()});
          u.weight += kv_tiles + ITEM_COST_TILES;
        }
      units.push_back(std::move(u));
    }
  }
  if (n_blocks == 0) {
    std::vector<std::vector<PrefillWork>> queue((size_t)xcds);
    if ((int)units.size() >= xcds) {
      std::vector<long> load((size_t)xcds, 0);
      std::vector<size_t> order(units.size());
      for (size_t i = 0; i < order.size(); ++i) order[i] = i;
      std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return units[a].weight > units[b].weight; });
      for (size_t ui : order) {
        const int x = (int)(std::min_element(load.begin(), load.end()) - load.begin());
        load[(size_t)x] += units[ui].weight;
        for (const Item& it : units[ui].items) queue[(size_t)x].push_back(it.w);
      }
    } else {
      size_t n = 0;
      for (Unit& u : units)
        for (Item& it : u.items) queue[n++ % (size_t)xcds].push_back(it.w);
    }
    size_t longest = 0;
    for (auto& qv : queue) longest = std::max(longest, qv.size());
    work.clear();
    chain.clear();
    for (size_t i = 0; i < longest; ++i)
      for (int x = 0; x < xcds; ++x) {          // workgroup i * xcds + x runs on XCD x
        chain.push_back((int32_t)work.size());
        if (i < queue[(size_t)x].size()) work.push_back(queue[(size_t)x][i]);
      }
    chain.push_back((int32_t)work.size());
    return;
  }
  if (n_blocks < xcds || n_blocks % xcds) xcds = 1;
  const int per_xcd = n_blocks / xcds;            // chains per XCD
  std::vector<std::vector<Item>> xq((size_t)xcds);
  if ((int)units.size() >= xcds) {
    std::vector<long> load((size_t)xcds, 0);
    std::vector<size_t> order(units.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return units[a].weight > units[b].weight; });
    for (size_t ui : order) {
      const int x = (int)(std::min_element(load.begin(), load.end()) - load.begin());
      load[(size_t)x] += units[ui].weight;
      xq[(size_t)x].insert(xq[(size_t)x].end(), units[ui].items.begin(), units[ui].items.end());
    }
  } else {
    size_t n = 0;
    for (Unit& u : units)
      for (Item& it : u.items) xq[n++ % (size_t)xcds].push_back(it);
  }
  std::vector<std::vector<Item>> chains((size_t)n_blocks);
  for (int x = 0; x < xcds; ++x) {
    // Unit after unit (in the order the XCD took them), each unit's items longest-first onto the chain
    // with the least load so far: every chain then holds about the same weight of EVERY unit, so the
    // chains of an XCD pass from one unit to the next at about the same time and the XCD's L2 has to
    // hold one or two units' K, V, not all of them.  (Dealt over all units at once the chains were as
    // well balanced in total, but drifted apart unit by unit, and K, V crossed HBM four times.)
    std::vector<Item>& items = xq[(size_t)x];
    std::vector<long> load((size_t)per_xcd, 0);
    size_t a = 0;
    while (a < items.size()) {
      size_t b = a;
      while (b < items.size() && items[b].unit == items[a].unit) ++b;
      std::stable_sort(items.begin() + (long)a, items.begin() + (long)b, [](const Item& p, const Item& q) { return p.weight > q.weight; });
      for (size_t i = a; i < b; ++i) {
        const int c = (int)(std::min_element(load.begin(), load.end()) - load.begin());
        load[(size_t)c] += items[i].weight;
        chains[(size_t)(c * xcds + x)].push_back(items[i]);          // workgroup id = chain slot * xcds + xcd
      }
      a = b;
    }
  }
  work.clear();
  chain.assign((size_t)n_blocks + 1, 0);
  for (int b = 0; b < n_blocks; ++b) {
    std::vector<Item>& ch = chains[(size_t)b];
    std::stable_sort(ch.begin(), ch.end(), [](const Item& a, const Item& c) { return a.unit < c.unit; });
    chain[(size_t)b] = (int32_t)work.size();
    for (const Item& it : ch) work.push_back(it.w);
  }
  chain[(size_t)n_blocks] = (int32_t)work.size();
}

}  // namespace spd
