// Host-side work list of the prefill kernel: which workgroup does what, and in which order.
#pragma once

#include <algorithm>
#include <vector>

#include "internal.h"

namespace spd {

// Workgroups are dispatched round-robin over the XCDs (workgroup i runs on XCD i % xcds), and each
// XCD has its own L2.  All workgroups that read the same K, V - the query tiles and head groups of
// one (request, KV head) "unit" - are therefore queued on the same XCD, one unit after the other,
// so that a unit's K, V is fetched into one L2 only and stays hot while its tiles run.  Inside a
// unit the causally heaviest tiles (largest tile index) go first.  Units are spread over the XCDs
// longest-first; with fewer units than XCDs the tiles themselves are dealt round-robin.
// prefix_lens (may be null): tokens of each request that precede its query rows; its keys / values
// then start at row kv_cu[r] of the K, V tensors (prefix + len rows per request), else at row0.
inline void build_prefill_work(const int32_t* cu_seqlens, const int32_t* prefix_lens, const int32_t* kv_cu, int n_req,
                               int H, int Hkv, int xcds, std::vector<PrefillWork>& out) {
  const int G = H / Hkv, hb = prefill_heads_per_block(G), bm = prefill_block_m(G), groups = G / hb;
  struct Unit { long weight; std::vector<PrefillWork> items; };
  std::vector<Unit> units;
  for (int r = 0; r < n_req; ++r) {
    const int32_t row0 = cu_seqlens[r], len = cu_seqlens[r + 1] - row0;
    const int32_t q_off = prefix_lens ? prefix_lens[r] : 0, kv_row0 = prefix_lens ? kv_cu[r] : row0;
    const int tiles = (len + bm - 1) / bm;
    for (int g = 0; g < Hkv; ++g) {
      Unit u{0, {}};
      for (int t = tiles - 1; t >= 0; --t)
        for (int hg = 0; hg < groups; ++hg) {
          u.items.push_back(PrefillWork{row0, len, t, g * G + hg * hb, kv_row0, q_off});
          u.weight += q_off + std::min<long>(len, (long)(t + 1) * bm);
        }
      units.push_back(std::move(u));
    }
  }
  std::vector<std::vector<PrefillWork>> queue((size_t)xcds);
  if ((int)units.size() >= xcds) {
    std::vector<long> load((size_t)xcds, 0);
    std::stable_sort(units.begin(), units.end(), [](const Unit& a, const Unit& b) { return a.weight > b.weight; });
    for (Unit& u : units) {
      const int x = (int)(std::min_element(load.begin(), load.end()) - load.begin());
      load[(size_t)x] += u.weight;
      queue[(size_t)x].insert(queue[(size_t)x].end(), u.items.begin(), u.items.end());
    }
  } else {
    size_t n = 0;
    for (Unit& u : units)
      for (PrefillWork& w : u.items) queue[n++ % (size_t)xcds].push_back(w);
  }
  size_t longest = 0;
  for (auto& qv : queue) longest = std::max(longest, qv.size());
  out.clear();
  out.reserve(longest * (size_t)xcds);
  for (size_t i = 0; i < longest; ++i)
    for (int x = 0; x < xcds; ++x)
      out.push_back(i < queue[(size_t)x].size() ? queue[(size_t)x][i] : PrefillWork{0, 0, 0, 0, 0, 0});
}

}  // namespace spd
